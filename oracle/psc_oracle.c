/*
 * CPU oracle for the polysemous-code search path -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, double-precision restatement of what the search path of
 * "Polysemous codes" (Douze, Jegou, Perronnin, ECCV 2016) computes.  It exists
 * so that the GPU library can be checked against something written from the
 * paper alone.  It shares no code, header, table or helper with the GPU
 * library, and nothing in the product path may call it: only the tests, the
 * smoke check and the benchmark's CPU-baseline leg load this file.
 *
 * Loops are scalar; the only parallelism is an OpenMP loop over queries (or
 * over database rows for encoding).  No blocking, no fusion, no early exit.
 *
 * Conventions (where the paper is silent these are this build's readings):
 *   - a product quantizer has m sub-quantizers of 256 centroids each; a code
 *     is m bytes, byte j = index chosen by sub-quantizer j (Section 3, first
 *     paragraphs; Section 3.1 "Notation", d = 8 bits per index);
 *   - the codebook is stored [m][256][dsub], already renumbered by the index
 *     assignment, so the search never sees the permutation (Section 1: the
 *     numeration of the centroids is re-ordered);
 *   - ADC distance = sum over sub-quantizers of the squared Euclidean distance
 *     between the query sub-vector and the selected centroid (the asymmetric
 *     estimator the paper cites in Section 4.2, "ADC");
 *   - Hamming distance is taken over all 8m bits of the code at once and a
 *     code is KEPT iff that distance is <= ht (Section 3.3 and Section 4.2
 *     "dual": codes whose distance is above the threshold are filtered out);
 *   - results are ordered by (distance, id) ascending, lower id first on equal
 *     distance; short lists are padded with id -1 and distance +infinity.
 *
 * Pins: see tests/test_oracle_*.py.
 * Parity unpinned: which local minimum k-means reaches on real data (train_pq,
 * ivf_train_coarse on the Python side; kmeans itself is pinned on small inputs
 * with a closed-form result) and which local minimum the simulated annealing
 * ends in (orc_anneal): nothing printed in the paper fixes them, so only their
 * invariants are pinned (objective never rises, result is a permutation,
 * incremental cost change = full recomputation, final loss below initial).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------- */
/* Hamming distance between two byte strings: number of differing bits.       */
/* Section 1 / Section 4.2 "binary": xor then count the set bits.             */
/* ------------------------------------------------------------------------- */
static int bits_set_in_byte(unsigned v)
{
    int c = 0;
    for (int b = 0; b < 8; ++b)
        c += (v >> b) & 1u;
    return c;
}

int orc_hamming(const uint8_t *a, const uint8_t *b, int nbytes)
{
    int h = 0;
    for (int j = 0; j < nbytes; ++j)
        h += bits_set_in_byte((unsigned)(a[j] ^ b[j]));
    return h;
}

/* All-pairs Hamming distances, out[q*n + i]; for small inputs only. */
void orc_hamming_matrix(const uint8_t *qcodes, int64_t nq, const uint8_t *codes, int64_t n,
                        int nbytes, int32_t *out)
{
    for (int64_t q = 0; q < nq; ++q)
        for (int64_t i = 0; i < n; ++i)
            out[q * n + i] = orc_hamming(qcodes + q * nbytes, codes + i * nbytes, nbytes);
}

/* ------------------------------------------------------------------------- */
/* Squared Euclidean distance, direct differences.                            */
/* ------------------------------------------------------------------------- */
static double sqdist(const double *a, const double *b, int n)
{
    double s = 0.0;
    for (int d = 0; d < n; ++d) {
        double t = a[d] - b[d];
        s += t * t;
    }
    return s;
}

/* ------------------------------------------------------------------------- */
/* PQ encoding: byte j of the code = nearest centroid of sub-quantizer j to   */
/* sub-vector j (lowest index on equal distance).                             */
/* x [n][D], cb [m][256][dsub], codes [n][m].                                 */
/* ------------------------------------------------------------------------- */
void orc_encode(const double *x, int64_t n, int D, int m, const double *cb, uint8_t *codes)
{
    int dsub = D / m;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        for (int j = 0; j < m; ++j) {
            const double *xj = x + i * D + j * dsub;
            int best = 0;
            double bestd = INFINITY;
            for (int c = 0; c < 256; ++c) {
                double dd = sqdist(xj, cb + ((int64_t)j * 256 + c) * dsub, dsub);
                if (dd < bestd) {
                    bestd = dd;
                    best = c;
                }
            }
            codes[i * m + j] = (uint8_t)best;
        }
    }
}

/* Nearest of ncent centroids for each row (lowest index on equal distance) and the
 * squared distance to it: the assignment step of Lloyd's k-means and of the coarse
 * quantizer.  x [n][d], cent [ncent][d]. */
void orc_nearest(const double *x, int64_t n, int d, const double *cent, int ncent,
                 int64_t *assign, double *dmin)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        int best = 0;
        double bestd = INFINITY;
        for (int c = 0; c < ncent; ++c) {
            double dd = sqdist(x + i * d, cent + (int64_t)c * d, d);
            if (dd < bestd) {
                bestd = dd;
                best = c;
            }
        }
        assign[i] = best;
        dmin[i] = bestd;
    }
}

/* Reconstruction of a code: concatenation of the selected centroids. */
void orc_decode(const uint8_t *codes, int64_t n, int D, int m, const double *cb, double *x)
{
    int dsub = D / m;
    for (int64_t i = 0; i < n; ++i)
        for (int j = 0; j < m; ++j)
            memcpy(x + i * D + j * dsub, cb + ((int64_t)j * 256 + codes[i * m + j]) * dsub,
                   sizeof(double) * dsub);
}

/* ------------------------------------------------------------------------- */
/* ADC look-up tables: lut[q][j][c] = || q_j - cb[j][c] ||^2.                 */
/* ------------------------------------------------------------------------- */
void orc_build_lut(const double *q, int64_t nq, int D, int m, const double *cb, double *lut)
{
    int dsub = D / m;
#pragma omp parallel for schedule(static)
    for (int64_t iq = 0; iq < nq; ++iq)
        for (int j = 0; j < m; ++j)
            for (int c = 0; c < 256; ++c)
                lut[(iq * m + j) * 256 + c] =
                    sqdist(q + iq * D + j * dsub, cb + ((int64_t)j * 256 + c) * dsub, dsub);
}

/* The query's own code: per sub-quantizer the index of the smallest table entry, */
/* lowest index on ties (identical to encoding the query with the codebook).      */
void orc_query_codes(const double *lut, int64_t nq, int m, uint8_t *qcodes)
{
    for (int64_t iq = 0; iq < nq; ++iq)
        for (int j = 0; j < m; ++j) {
            const double *row = lut + (iq * m + j) * 256;
            int best = 0;
            for (int c = 1; c < 256; ++c)
                if (row[c] < row[best])
                    best = c;
            qcodes[iq * m + j] = (uint8_t)best;
        }
}

/* ------------------------------------------------------------------------- */
/* The "dual" scan (Section 3.3, Section 4.2):                                */
/*   for every database code: Hamming distance to the query's code; codes     */
/*   with distance > ht are dropped; survivors get their ADC distance (sum of */
/*   m table entries, j ascending); survivors are sorted by (distance, id)    */
/*   and the first k are returned.                                            */
/* ------------------------------------------------------------------------- */
typedef struct {
    double dist;
    int64_t id;
} cand_t;

static int cand_cmp(const void *pa, const void *pb)
{
    const cand_t *a = (const cand_t *)pa, *b = (const cand_t *)pb;
    if (a->dist < b->dist) return -1;
    if (a->dist > b->dist) return 1;
    if (a->id < b->id) return -1;
    if (a->id > b->id) return 1;
    return 0;
}

/*
 * (Arguments of orc_scan and orc_scan_filtered.)
 * lut [nq][m][256] (double), qcodes [nq][m], codes [n][m].
 * ext_ids: NULL -> the id of database row i is i; else the id is ext_ids[i].
 * skip_id: NULL -> nothing skipped; else for query q the row whose id equals
 *          skip_id[q] is never returned (k-NN-graph mode: a vector is not its
 *          own neighbour).  A skipped row is still counted as a survivor.
 * ids, dists [nq][k]; nsurv [nq] (may be NULL) = number of codes with
 * Hamming distance <= ht.
 * surv_bitmap (may be NULL): [nq][n] bytes, 1 where the code survives.
 * Returns 0, or -1 on allocation failure.
 */
/* The alternative filter of Section 3.3 (second paragraph; "disidx" in Section 4.2): how many   */
/* sub-quantizers give an index different from the query's -- a Hamming distance between vectors */
/* of indexes, not of bits.                                                                      */
int orc_disidx(const uint8_t *a, const uint8_t *b, int nbytes)
{
    int h = 0;
    for (int j = 0; j < nbytes; ++j)
        h += (a[j] != b[j]);
    return h;
}

int orc_scan_filtered(int m, const double *lut, const uint8_t *qcodes, int64_t nq, const uint8_t *codes,
                      int64_t n, int filter, int ht, int k, const int64_t *ext_ids, const int64_t *skip_id,
                      int64_t *ids, double *dists, int64_t *nsurv, uint8_t *surv_bitmap);

int orc_scan(int m, const double *lut, const uint8_t *qcodes, int64_t nq, const uint8_t *codes,
             int64_t n, int ht, int k, const int64_t *ext_ids, const int64_t *skip_id,
             int64_t *ids, double *dists, int64_t *nsurv, uint8_t *surv_bitmap)
{
    return orc_scan_filtered(m, lut, qcodes, nq, codes, n, 0, ht, k, ext_ids, skip_id, ids, dists, nsurv,
                             surv_bitmap);
}

/* filter = 0: Hamming distance over the bits (the polysemous filter, "dual");                   */
/* filter = 1: number of differing indexes ("disidx"), kept iff that number is <= ht.            */
int orc_scan_filtered(int m, const double *lut, const uint8_t *qcodes, int64_t nq, const uint8_t *codes,
                      int64_t n, int filter, int ht, int k, const int64_t *ext_ids, const int64_t *skip_id,
                      int64_t *ids, double *dists, int64_t *nsurv, uint8_t *surv_bitmap)
{
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t q = 0; q < nq; ++q) {
        cand_t *cand = (cand_t *)malloc(sizeof(cand_t) * (size_t)(n > 0 ? n : 1));
        if (!cand) {
#pragma omp atomic write
            failed = 1;
            continue;
        }
        const uint8_t *qc = qcodes + q * m;
        const double *tab = lut + q * m * 256;
        int64_t ns = 0, nc = 0;
        for (int64_t i = 0; i < n; ++i) {
            const uint8_t *code = codes + i * m;
            int h = filter == 1 ? orc_disidx(qc, code, m) : orc_hamming(qc, code, m);
            int keep = (h <= ht);
            if (surv_bitmap)
                surv_bitmap[q * n + i] = (uint8_t)keep;
            if (!keep)
                continue;
            ++ns;
            int64_t id = ext_ids ? ext_ids[i] : i;
            if (skip_id && id == skip_id[q])
                continue;
            double d = 0.0;
            for (int j = 0; j < m; ++j)
                d += tab[j * 256 + code[j]];
            cand[nc].dist = d;
            cand[nc].id = id;
            ++nc;
        }
        qsort(cand, (size_t)nc, sizeof(cand_t), cand_cmp);
        for (int r = 0; r < k; ++r) {
            if (r < nc) {
                ids[q * k + r] = cand[r].id;
                dists[q * k + r] = cand[r].dist;
            } else {
                ids[q * k + r] = -1;
                dists[q * k + r] = INFINITY;
            }
        }
        if (nsurv)
            nsurv[q] = ns;
        free(cand);
    }
    return failed ? -1 : 0;
}

/* ------------------------------------------------------------------------- */
/* Inverted-file search with residual codes (Section 2 "Non-exhaustive        */
/* search", Section 4.3):                                                     */
/*   1. the nprobe coarse centroids nearest to the query (exact squared L2,   */
/*      lower list number on ties);                                           */
/*   2. for each probed list l: residual r = q - coarse[l]; tables from r;    */
/*      query code = code of r; Hamming filter + ADC over the list's codes;   */
/*   3. one ranking over the union of the probed lists; ids come from the     */
/*      list's id array.                                                      */
/* offsets [nlist+1], codes [N][m] grouped by list, list_ids [N] (int32).     */
/* probed [nq][nprobe] (may be NULL) receives the probed list numbers in      */
/* ascending coarse distance.                                                 */
/* ------------------------------------------------------------------------- */
typedef struct {
    double dist;
    int list;
} coarse_t;

static int coarse_cmp(const void *pa, const void *pb)
{
    const coarse_t *a = (const coarse_t *)pa, *b = (const coarse_t *)pb;
    if (a->dist < b->dist) return -1;
    if (a->dist > b->dist) return 1;
    return (a->list > b->list) - (a->list < b->list);
}

/* probed_in (may be NULL) [nq][nprobe]: take these lists instead of ranking the coarse        */
/* centroids; qcodes_in (may be NULL) [nq][nprobe][m]: take these bit strings for the filter   */
/* instead of the arg-min of the residual tables.  Both exist so that a float32 implementation  */
/* whose near-ties fall the other way can be checked on identical decisions.                   */
int orc_ivf_search(int D, int m, const double *cb, const double *coarse, int nlist,
                   const int64_t *offsets, const uint8_t *codes, const int32_t *list_ids,
                   const double *queries, int64_t nq, int nprobe, int ht, int k,
                   const int32_t *probed_in, const uint8_t *qcodes_in,
                   int64_t *ids, double *dists, int64_t *nsurv, int32_t *probed, double *coarse_d)
{
    int dsub = D / m;
    if (nprobe > nlist)
        nprobe = nlist;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t q = 0; q < nq; ++q) {
        const double *qv = queries + q * D;
        coarse_t *cl = (coarse_t *)malloc(sizeof(coarse_t) * (size_t)nlist);
        double *res = (double *)malloc(sizeof(double) * (size_t)D);
        double *tab = (double *)malloc(sizeof(double) * (size_t)m * 256);
        uint8_t *qc = (uint8_t *)malloc((size_t)m);
        int64_t total = 0;
        if (cl) {
            for (int l = 0; l < nlist; ++l) {
                cl[l].dist = sqdist(qv, coarse + (int64_t)l * D, D);
                cl[l].list = l;
                if (coarse_d)
                    coarse_d[q * nlist + l] = cl[l].dist;
            }
            qsort(cl, (size_t)nlist, sizeof(coarse_t), coarse_cmp);
            if (probed_in)
                for (int p = 0; p < nprobe; ++p)
                    cl[p].list = probed_in[q * nprobe + p];
            for (int p = 0; p < nprobe; ++p)
                total += offsets[cl[p].list + 1] - offsets[cl[p].list];
        }
        cand_t *cand = (cand_t *)malloc(sizeof(cand_t) * (size_t)(total > 0 ? total : 1));
        if (!cl || !res || !tab || !qc || !cand) {
#pragma omp atomic write
            failed = 1;
            free(cl); free(res); free(tab); free(qc); free(cand);
            continue;
        }
        int64_t ns = 0, nc = 0;
        for (int p = 0; p < nprobe; ++p) {
            int l = cl[p].list;
            if (probed)
                probed[q * nprobe + p] = l;
            for (int d = 0; d < D; ++d)
                res[d] = qv[d] - coarse[(int64_t)l * D + d];
            for (int j = 0; j < m; ++j) {
                int best = 0;
                for (int c = 0; c < 256; ++c) {
                    tab[j * 256 + c] =
                        sqdist(res + j * dsub, cb + ((int64_t)j * 256 + c) * dsub, dsub);
                    if (tab[j * 256 + c] < tab[j * 256 + best])
                        best = c;
                }
                qc[j] = qcodes_in ? qcodes_in[(q * nprobe + p) * m + j] : (uint8_t)best;
            }
            for (int64_t i = offsets[l]; i < offsets[l + 1]; ++i) {
                const uint8_t *code = codes + i * m;
                if (orc_hamming(qc, code, m) > ht)
                    continue;
                ++ns;
                double dd = 0.0;
                for (int j = 0; j < m; ++j)
                    dd += tab[j * 256 + code[j]];
                cand[nc].dist = dd;
                cand[nc].id = list_ids[i];
                ++nc;
            }
        }
        qsort(cand, (size_t)nc, sizeof(cand_t), cand_cmp);
        for (int r = 0; r < k; ++r) {
            if (r < nc) {
                ids[q * k + r] = cand[r].id;
                dists[q * k + r] = cand[r].dist;
            } else {
                ids[q * k + r] = -1;
                dists[q * k + r] = INFINITY;
            }
        }
        if (nsurv)
            nsurv[q] = ns;
        free(cl); free(res); free(tab); free(qc); free(cand);
    }
    return failed ? -1 : 0;
}

/* ------------------------------------------------------------------------- */
/* Inverted multi-index (Section 2 "Non-exhaustive search", Section 4.3 and   */
/* the caption of Table 2): the coarse level is a product quantizer -- the    */
/* first half of a vector is quantized with K1 centroids, the second half     */
/* with K2 -- so there are K1*K2 cells, cell (a,b) = number a*K2 + b, with    */
/* centroid (coarse1[a], coarse2[b]).  A query visits the cells in            */
/* non-decreasing order of its squared distance to the cell centroid, which   */
/* is d1[a] + d2[b] (lower cell number first on equal distance), until        */
/* max_lists cells have been taken or the cells taken so far hold max_codes   */
/* codes or more (max_codes <= 0: no such cap; the cell that reaches the cap   */
/* is still scanned whole; an empty cell counts as a visited cell).  Inside a  */
/* cell everything is as in orc_ivf_search: residual to the cell centroid,     */
/* tables and bit string from the residual, Hamming filter, ADC; one ranking   */
/* over all visited cells.                                                     */
/* offsets [K1*K2+1]; cells [nq][max_lists] (may be NULL) receives the cells    */
/* taken, in order, padded with -1; ncodes [nq] (may be NULL) the codes they    */
/* hold.  cells_in (may be NULL) [nq][max_lists], padded with -1: take exactly  */
/* these cells instead; qcodes_in (may be NULL) [nq][max_lists][m]: these bit    */
/* strings.                                                                    */
/* ------------------------------------------------------------------------- */
int orc_imi_search(int D, int m, const double *cb, const double *coarse1, int K1, const double *coarse2, int K2,
                   const int64_t *offsets, const uint8_t *codes, const int32_t *list_ids,
                   const double *queries, int64_t nq, int max_lists, int64_t max_codes, int ht, int k,
                   const int32_t *cells_in, const uint8_t *qcodes_in,
                   int64_t *ids, double *dists, int64_t *nsurv, int32_t *cells, int64_t *ncodes)
{
    int dsub = D / m, half = D / 2;
    int64_t ncell = (int64_t)K1 * K2;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t q = 0; q < nq; ++q) {
        const double *qv = queries + q * D;
        coarse_t *cl = (coarse_t *)malloc(sizeof(coarse_t) * (size_t)ncell);
        int32_t *take = (int32_t *)malloc(sizeof(int32_t) * (size_t)(max_lists > 0 ? max_lists : 1));
        double *res = (double *)malloc(sizeof(double) * (size_t)D);
        double *tab = (double *)malloc(sizeof(double) * (size_t)m * 256);
        uint8_t *qc = (uint8_t *)malloc((size_t)m);
        int ntake = 0;
        int64_t total = 0;
        if (cl && take) {
            if (cells_in) {
                for (int p = 0; p < max_lists && cells_in[q * max_lists + p] >= 0; ++p) {
                    take[ntake++] = cells_in[q * max_lists + p];
                    total += offsets[take[ntake - 1] + 1] - offsets[take[ntake - 1]];
                }
            } else {
                for (int a = 0; a < K1; ++a) {
                    double d1 = sqdist(qv, coarse1 + (int64_t)a * half, half);
                    for (int b = 0; b < K2; ++b) {
                        cl[(int64_t)a * K2 + b].dist = d1 + sqdist(qv + half, coarse2 + (int64_t)b * half, half);
                        cl[(int64_t)a * K2 + b].list = (int)((int64_t)a * K2 + b);
                    }
                }
                qsort(cl, (size_t)ncell, sizeof(coarse_t), coarse_cmp);
                for (int64_t t = 0; t < ncell; ++t) {
                    if (ntake == max_lists || (max_codes > 0 && total >= max_codes))
                        break;
                    take[ntake++] = cl[t].list;
                    total += offsets[cl[t].list + 1] - offsets[cl[t].list];
                }
            }
        }
        cand_t *cand = (cand_t *)malloc(sizeof(cand_t) * (size_t)(total > 0 ? total : 1));
        if (!cl || !take || !res || !tab || !qc || !cand) {
#pragma omp atomic write
            failed = 1;
            free(cl); free(take); free(res); free(tab); free(qc); free(cand);
            continue;
        }
        int64_t ns = 0, nc = 0;
        for (int p = 0; p < max_lists; ++p)
            if (cells)
                cells[q * max_lists + p] = p < ntake ? take[p] : -1;
        for (int p = 0; p < ntake; ++p) {
            int cell = take[p], a = cell / K2, b = cell % K2;
            for (int d = 0; d < half; ++d) {
                res[d] = qv[d] - coarse1[(int64_t)a * half + d];
                res[half + d] = qv[half + d] - coarse2[(int64_t)b * half + d];
            }
            for (int j = 0; j < m; ++j) {
                int best = 0;
                for (int c = 0; c < 256; ++c) {
                    tab[j * 256 + c] = sqdist(res + j * dsub, cb + ((int64_t)j * 256 + c) * dsub, dsub);
                    if (tab[j * 256 + c] < tab[j * 256 + best])
                        best = c;
                }
                qc[j] = qcodes_in ? qcodes_in[(q * max_lists + p) * m + j] : (uint8_t)best;
            }
            for (int64_t i = offsets[cell]; i < offsets[cell + 1]; ++i) {
                const uint8_t *code = codes + i * m;
                if (orc_hamming(qc, code, m) > ht)
                    continue;
                ++ns;
                double dd = 0.0;
                for (int j = 0; j < m; ++j)
                    dd += tab[j * 256 + code[j]];
                cand[nc].dist = dd;
                cand[nc].id = list_ids[i];
                ++nc;
            }
        }
        qsort(cand, (size_t)nc, sizeof(cand_t), cand_cmp);
        for (int r = 0; r < k; ++r) {
            ids[q * k + r] = r < nc ? cand[r].id : -1;
            dists[q * k + r] = r < nc ? cand[r].dist : INFINITY;
        }
        if (nsurv)
            nsurv[q] = ns;
        if (ncodes)
            ncodes[q] = total;
        free(cl); free(take); free(res); free(tab); free(qc); free(cand);
    }
    return failed ? -1 : 0;
}

/* ------------------------------------------------------------------------- */
/* Exact k nearest neighbours on raw vectors (ground truth for recall@R,      */
/* Section 4.1): squared L2, (distance, id) ascending.  skip_self != 0: row q */
/* of the queries is database row q and is not its own neighbour.             */
/* ------------------------------------------------------------------------- */
int orc_exact_knn(const double *x, int64_t n, const double *queries, int64_t nq, int D, int k,
                  int skip_self, int64_t *ids, double *dists)
{
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t q = 0; q < nq; ++q) {
        cand_t *cand = (cand_t *)malloc(sizeof(cand_t) * (size_t)(n > 0 ? n : 1));
        if (!cand) {
#pragma omp atomic write
            failed = 1;
            continue;
        }
        int64_t nc = 0;
        for (int64_t i = 0; i < n; ++i) {
            if (skip_self && i == q)
                continue;
            cand[nc].dist = sqdist(queries + q * D, x + i * D, D);
            cand[nc].id = i;
            ++nc;
        }
        qsort(cand, (size_t)nc, sizeof(cand_t), cand_cmp);
        for (int r = 0; r < k; ++r) {
            ids[q * k + r] = r < nc ? cand[r].id : -1;
            dists[q * k + r] = r < nc ? cand[r].dist : INFINITY;
        }
        free(cand);
    }
    return failed ? -1 : 0;
}

/* ------------------------------------------------------------------------- */
/* Index assignment by simulated annealing on the weighted distance-estimator */
/* loss (Section 3.1, weighted objective; Section 3.2, the annealing loop).   */
/*                                                                            */
/*   d_ij  = Euclidean distance between centroids i and j                     */
/*   mu, sigma = mean and standard deviation of d_ij over ordered pairs i!=j  */
/*   f(x)  = sqrt(nbit)/(2 sigma) * (x - mu) + nbit/2        (linear map)     */
/*   w(u)  = alpha^u                                                          */
/*   L(pi) = sum_{i,j} w(f(d_ij)) * [ h(pi_i, pi_j) - f(d_ij) ]^2             */
/*                                                                            */
/* pi[i] is the new nbit-bit index of centroid i.                             */
/* ------------------------------------------------------------------------- */
#define NCENT 256

void orc_centroid_distances(const double *cent, int dsub, double *dmat /*256x256*/)
{
    for (int i = 0; i < NCENT; ++i)
        for (int j = 0; j < NCENT; ++j)
            dmat[i * NCENT + j] = sqrt(sqdist(cent + (int64_t)i * dsub, cent + (int64_t)j * dsub, dsub));
}

void orc_distance_stats(const double *dmat, double *mu, double *sigma)
{
    double s = 0.0, s2 = 0.0;
    int64_t cnt = 0;
    for (int i = 0; i < NCENT; ++i)
        for (int j = 0; j < NCENT; ++j)
            if (i != j) {
                s += dmat[i * NCENT + j];
                ++cnt;
            }
    double mean = s / (double)cnt;
    for (int i = 0; i < NCENT; ++i)
        for (int j = 0; j < NCENT; ++j)
            if (i != j) {
                double t = dmat[i * NCENT + j] - mean;
                s2 += t * t;
            }
    *mu = mean;
    *sigma = sqrt(s2 / (double)cnt);
}

/* The linear map f of Section 3.1 for nbit-bit indices. */
double orc_f(double x, double mu, double sigma, int nbit)
{
    return sqrt((double)nbit) / (2.0 * sigma) * (x - mu) + (double)nbit / 2.0;
}

/* target[i][j] = f(d_ij), weight[i][j] = alpha^target[i][j]. */
void orc_targets_weights(const double *dmat, double mu, double sigma, double alpha, int nbit,
                         double *target, double *weight)
{
    for (int i = 0; i < NCENT * NCENT; ++i) {
        target[i] = orc_f(dmat[i], mu, sigma, nbit);
        weight[i] = pow(alpha, target[i]);
    }
}

static int hamming_idx(unsigned a, unsigned b)
{
    return bits_set_in_byte((a ^ b) & 0xffu);
}

/* Full evaluation of the weighted loss, O(2^{2d}). */
double orc_polyd_loss(const double *target, const double *weight, const uint8_t *pi)
{
    double L = 0.0;
    for (int i = 0; i < NCENT; ++i)
        for (int j = 0; j < NCENT; ++j) {
            double e = (double)hamming_idx(pi[i], pi[j]) - target[i * NCENT + j];
            L += weight[i * NCENT + j] * e * e;
        }
    return L;
}

/* Loss change if entries a and b of pi were swapped, O(2^d): only the terms
 * with exactly one index in {a,b} change (the pair (a,b) itself keeps its
 * Hamming distance).  Each unordered pair appears twice in the full sum, and
 * target/weight are symmetric, hence the factor 2. */
double orc_swap_delta(const double *target, const double *weight, const uint8_t *pi, int a, int b)
{
    double delta = 0.0;
    for (int k = 0; k < NCENT; ++k) {
        if (k == a || k == b)
            continue;
        double ha = (double)hamming_idx(pi[a], pi[k]);
        double hb = (double)hamming_idx(pi[b], pi[k]);
        double ta = target[a * NCENT + k], tb = target[b * NCENT + k];
        double wa = weight[a * NCENT + k], wb = weight[b * NCENT + k];
        /* after the swap centroid a carries pi[b] and centroid b carries pi[a] */
        delta += wa * ((hb - ta) * (hb - ta) - (ha - ta) * (ha - ta));
        delta += wb * ((ha - tb) * (ha - tb) - (hb - tb) * (hb - tb));
    }
    return 2.0 * delta;
}

/* Counter-based random numbers: draw number c under `seed` is the SplitMix64
 * output function applied to seed + (c+1)*golden-gamma.  The library under
 * test implements the same published generator so that, given the same seed,
 * both anneal along the same sequence of proposals. */
static uint64_t draw_u64(uint64_t seed, uint64_t c)
{
    uint64_t z = seed + (c + 1) * 0x9E3779B97F4A7C15ULL;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

uint64_t orc_draw_u64(uint64_t seed, uint64_t c) { return draw_u64(seed, c); }

/*
 * Simulated annealing (Section 3.2): start from the identity, temperature t0;
 * each iteration draws i != j, computes the loss change of swapping pi[i] and
 * pi[j], accepts when the change is negative or, otherwise, with probability
 * t; then t <- t * t_decay.
 * Iteration it uses draws 3it (i), 3it+1 (j), 3it+2 (acceptance).
 * pi_out [256]; loss_trace (may be NULL) [n_iter+1] = loss before each
 * iteration and after the last one, tracked through the accepted changes.
 */
void orc_anneal(const double *cent, int dsub, int64_t n_iter, double t0, double t_decay,
                double alpha, uint64_t seed, uint8_t *pi_out, double *loss_init,
                double *loss_final, double *loss_trace)
{
    const int nbit = 8;
    double *dmat = (double *)malloc(sizeof(double) * NCENT * NCENT);
    double *target = (double *)malloc(sizeof(double) * NCENT * NCENT);
    double *weight = (double *)malloc(sizeof(double) * NCENT * NCENT);
    double mu, sigma;
    orc_centroid_distances(cent, dsub, dmat);
    orc_distance_stats(dmat, &mu, &sigma);
    orc_targets_weights(dmat, mu, sigma, alpha, nbit, target, weight);

    uint8_t pi[NCENT];
    for (int i = 0; i < NCENT; ++i)
        pi[i] = (uint8_t)i;
    double L = orc_polyd_loss(target, weight, pi);
    if (loss_init)
        *loss_init = L;
    double t = t0;
    for (int64_t it = 0; it < n_iter; ++it) {
        if (loss_trace)
            loss_trace[it] = L;
        int i = (int)(draw_u64(seed, 3 * (uint64_t)it) % NCENT);
        int j = (int)((i + 1 + draw_u64(seed, 3 * (uint64_t)it + 1) % (NCENT - 1)) % NCENT);
        double u = (double)(draw_u64(seed, 3 * (uint64_t)it + 2) >> 11) * (1.0 / 9007199254740992.0);
        double dC = orc_swap_delta(target, weight, pi, i, j);
        if (dC < 0.0 || u < t) {
            uint8_t tmp = pi[i];
            pi[i] = pi[j];
            pi[j] = tmp;
            L += dC;
        }
        t *= t_decay;
    }
    if (loss_trace)
        loss_trace[n_iter] = L;
    if (loss_final)
        *loss_final = orc_polyd_loss(target, weight, pi);
    memcpy(pi_out, pi, NCENT);
    free(dmat);
    free(target);
    free(weight);
}

/* Renumber one sub-quantizer: new row pi[i] := old row i. */
void orc_apply_assignment(const double *cent_in, int dsub, const uint8_t *pi, double *cent_out)
{
    for (int i = 0; i < NCENT; ++i)
        memcpy(cent_out + (int64_t)pi[i] * dsub, cent_in + (int64_t)i * dsub, sizeof(double) * dsub);
}


/* ------------------------------------------------------------------------- */
/* Ranking loss (Section 3.1, "Ranking loss") and its annealing.              */
/*                                                                            */
/*   rank(i,j)  = position of j in the list of centroids ordered by distance  */
/*                to i: the number of centroids k with d_ik < d_ij.  Centroid  */
/*                i itself (d_ii = 0) is one of them, so the nearest other     */
/*                centroid has rank 1.  (The printed formula counts the        */
/*                centroids FARTHER than j; the text next to it calls it the   */
/*                rank of j among the neighbours of i and uses it to weigh     */
/*                far-away j down, which only the count of nearer ones does.)  */
/*   r_pi(i,j)  = number of k that are farther from i than j by centroid       */
/*                distance but nearer than j by Hamming distance of indexes:   */
/*                sum_k [d_ij < d_ik] [h(pi_i,pi_j) > h(pi_i,pi_k)]            */
/*   alpha_r    = 1/r,   ell_r = alpha_1 + ... + alpha_r  (ell_0 = 0)          */
/*   L(pi)      = sum_{i != j} alpha_rank(i,j) * ell_{r_pi(i,j)}               */
/* ------------------------------------------------------------------------- */
void orc_neighbour_ranks(const double *dmat, int32_t *rank /*256x256*/)
{
    for (int i = 0; i < NCENT; ++i)
        for (int j = 0; j < NCENT; ++j) {
            int r = 0;
            for (int k = 0; k < NCENT; ++k)
                r += dmat[i * NCENT + k] < dmat[i * NCENT + j];
            rank[i * NCENT + j] = r;
        }
}

int orc_rank_violations(const double *dmat, const uint8_t *pi, int i, int j)
{
    int r = 0;
    int hij = hamming_idx(pi[i], pi[j]);
    for (int k = 0; k < NCENT; ++k)
        r += (dmat[i * NCENT + j] < dmat[i * NCENT + k]) && (hij > hamming_idx(pi[i], pi[k]));
    return r;
}

double orc_ell(int r)
{
    double s = 0.0;
    for (int t = 1; t <= r; ++t)
        s += 1.0 / (double)t;
    return s;
}

/* Full evaluation, O(2^{3d}).  Pairs with rank 0 (j = i, or an exact duplicate of centroid i) have */
/* no weight alpha_0 and are left out. */
double orc_polyr_loss(const double *dmat, const int32_t *rank, const uint8_t *pi)
{
    double L = 0.0;
    for (int i = 0; i < NCENT; ++i)
        for (int j = 0; j < NCENT; ++j) {
            if (j == i || rank[i * NCENT + j] == 0)
                continue;
            L += orc_ell(orc_rank_violations(dmat, pi, i, j)) / (double)rank[i * NCENT + j];
        }
    return L;
}

/* Loss change if entries a and b of pi were swapped, O(2^{2d}): for a pair (i,j) with i, j outside */
/* {a,b} only the two terms k = a and k = b of r_pi(i,j) can change; pairs with i or j in {a,b} are */
/* counted afresh.  Pairs whose count does not change contribute exactly nothing.                  */
double orc_polyr_swap_delta(const double *dmat, const int32_t *rank, const uint8_t *pi, int a, int b)
{
    uint8_t pj[NCENT];
    memcpy(pj, pi, NCENT);
    pj[a] = pi[b];
    pj[b] = pi[a];
    double delta = 0.0;
    for (int i = 0; i < NCENT; ++i)
        for (int j = 0; j < NCENT; ++j) {
            if (j == i || rank[i * NCENT + j] == 0)
                continue;
            int r_old, r_new;
            if (i == a || i == b || j == a || j == b) {
                r_old = orc_rank_violations(dmat, pi, i, j);
                r_new = orc_rank_violations(dmat, pj, i, j);
                if (r_old == r_new)
                    continue;
            } else {
                /* only k = a and k = b see another index; h(pi_i, pi_j) is unchanged */
                int hij = hamming_idx(pi[i], pi[j]);
                int fa = dmat[i * NCENT + j] < dmat[i * NCENT + a];
                int fb = dmat[i * NCENT + j] < dmat[i * NCENT + b];
                int before = (fa && hij > hamming_idx(pi[i], pi[a])) + (fb && hij > hamming_idx(pi[i], pi[b]));
                int after = (fa && hij > hamming_idx(pi[i], pj[a])) + (fb && hij > hamming_idx(pi[i], pj[b]));
                if (before == after)
                    continue;
                r_old = orc_rank_violations(dmat, pi, i, j);
                r_new = r_old - before + after;
            }
            delta += (orc_ell(r_new) - orc_ell(r_old)) / (double)rank[i * NCENT + j];
        }
    return delta;
}

/* The annealing of Section 3.2 on the ranking loss: same loop, same random draws as orc_anneal. */
void orc_anneal_ranking(const double *cent, int dsub, int64_t n_iter, double t0, double t_decay,
                        uint64_t seed, uint8_t *pi_out, double *loss_init, double *loss_final,
                        double *loss_trace)
{
    double *dmat = (double *)malloc(sizeof(double) * NCENT * NCENT);
    int32_t *rank = (int32_t *)malloc(sizeof(int32_t) * NCENT * NCENT);
    orc_centroid_distances(cent, dsub, dmat);
    orc_neighbour_ranks(dmat, rank);
    uint8_t pi[NCENT];
    for (int i = 0; i < NCENT; ++i)
        pi[i] = (uint8_t)i;
    double L = orc_polyr_loss(dmat, rank, pi);
    if (loss_init)
        *loss_init = L;
    double t = t0;
    for (int64_t it = 0; it < n_iter; ++it) {
        if (loss_trace)
            loss_trace[it] = L;
        int i = (int)(draw_u64(seed, 3 * (uint64_t)it) % NCENT);
        int j = (int)((i + 1 + draw_u64(seed, 3 * (uint64_t)it + 1) % (NCENT - 1)) % NCENT);
        double u = (double)(draw_u64(seed, 3 * (uint64_t)it + 2) >> 11) * (1.0 / 9007199254740992.0);
        double dC = orc_polyr_swap_delta(dmat, rank, pi, i, j);
        if (dC < 0.0 || u < t) {
            uint8_t tmp = pi[i];
            pi[i] = pi[j];
            pi[j] = tmp;
            L += dC;
        }
        t *= t_decay;
    }
    if (loss_trace)
        loss_trace[n_iter] = L;
    if (loss_final)
        *loss_final = orc_polyr_loss(dmat, rank, pi);
    memcpy(pi_out, pi, NCENT);
    free(dmat);
    free(rank);
}
