/*
 * psc.h -- C ABI of the polysemous-code search library for AMD MI355X (gfx950).
 *
 * The library implements the search path of "Polysemous codes" (Douze, Jegou,
 * Perronnin, ECCV 2016): a scan over product-quantizer codes in which every
 * code is first compared as a bit string with the query's own code (Hamming
 * distance, Section 3.3 / Section 4.2 "dual"), codes farther than a threshold
 * are dropped, the survivors are scored with the asymmetric distance estimator
 * (a sum of per-sub-quantizer table entries, Section 4.2 "ADC") and the best k
 * per query are returned; plus the inverted-file variant with residual codes
 * (Section 4.3) and the all-against-all k-NN-graph mode (Section 5).
 *
 * General rules
 *   - Pointers named *_dev are device (HBM) pointers, *_host are host pointers.
 *     Every buffer is owned by the caller; the library allocates no device
 *     memory on the search path (workspaces are passed in and sized by the
 *     *_workspace_bytes functions).  The one exception is the index's own device
 *     image (codebook, coarse centroids, per-list tables): the first device call
 *     after the codebook or the coarse centroids changed uploads it, which
 *     allocates and blocks (it waits for all earlier work of the device, so that
 *     no kernel still reads the image it replaces).  psc_prepare does that upload
 *     ahead of time.
 *   - An index may be used from several host threads; training and set_* calls
 *     must not run concurrently with other calls on the same index.
 *   - All arrays are dense, row-major.  A product quantizer has m sub-quantizers
 *     (m = 8 or 16) of exactly 256 centroids; a code is m bytes, byte j holding
 *     the index chosen by sub-quantizer j.  Code arrays and query-code arrays
 *     must be 16-byte aligned.
 *   - Device work is enqueued on `stream` (a hipStream_t, 0 = the null stream)
 *     and the call returns without waiting, except where stated.
 *   - Return value: 0 on success, negative on failure:
 *        PSC_EINVAL  invalid argument (null pointer, unsupported m, k or size,
 *                    misaligned codes, workspace too small)
 *        PSC_ESTATE  the index lacks what the call needs (no codebook, no lists)
 *        PSC_EHIP    a HIP call failed
 *        PSC_ENOMEM  host allocation failed
 *     psc_last_error() gives a message for the last failure on the calling thread.
 *     Nothing throws or aborts across this boundary.
 *   - n = 0 or nq = 0 succeed; with n = 0 every result row is padding.
 */
#ifndef PSC_H
#define PSC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PSC_OK 0
#define PSC_EINVAL (-1)
#define PSC_ESTATE (-2)
#define PSC_EHIP (-3)
#define PSC_ENOMEM (-4)

#define PSC_MAX_K 1024

typedef struct psc_index psc_index; /* opaque: codebook (host + device copy), coarse centroids, list views */
typedef void *psc_stream;           /* hipStream_t */

/* Library version (major*10000 + minor*100 + patch). */
int psc_version(void);
/* Message describing the last failure on this thread ("" if none). */
const char *psc_last_error(void);

/* ------------------------------------------------------------------ lifecycle */
/* New index for dim-dimensional vectors and m sub-quantizers (m in {8,16},
 * dim % m == 0, dim/m one of 1,2,4,6,8,12,16,24,32,48,64).  Touches no device: the codebook is
 * copied to the current HIP device by the first device operation that needs it. */
int psc_create(psc_index **out, int dim, int m);
void psc_destroy(psc_index *idx);

/* ------------------------------------------------------------------ training (host side, synchronous) */
/* Product quantizer (Section 3, opening): one k-means with 256 centroids per
 * sub-space, `iters` Lloyd iterations, on n >= 256 training vectors
 * x_host [n][dim] (float32).  Replaces the codebook.
 * Start of sub-quantizer j: 256 distinct rows by a partial Fisher-Yates shuffle of the row
 * numbers 0..n-1: for c = 0..255, swap entry c with entry c + (draw c of SplitMix64 stream
 * seed + j) mod (n - c); row c of the start is the sub-vector of entry c.  (The coarse
 * quantizer's training starts the same way, nlist rows from stream `seed`.)
 * An empty cell takes the member of the (currently) most populated cell that lies farthest from
 * that cell's centroid. */
int psc_train_pq(psc_index *idx, const float *x_host, int64_t n, int iters, uint64_t seed);

/* The same training on the current device (Section 3, opening): x_dev [n][dim] float32 in device
 * memory, 256 <= n < 2^31.  start = PSC_START_SEEDED draws the same 256 starting rows per
 * sub-quantizer as psc_train_pq does for that seed; PSC_START_CURRENT continues from the index's
 * codebook (seed unused).  Each iteration assigns every sub-vector to its nearest centroid
 * (float32, coordinates in ascending order, lowest index on equal distance), replaces every centroid
 * by the mean of its members (sums in double precision) and refills an empty cell with the member
 * of the (currently) most populated cell that lies farthest from that cell's centroid (lowest row
 * on ties; the donor cell's mean still counts that member in the same iteration).
 * objective_out_host (may be NULL) [iters][m] receives, per iteration and sub-quantizer, the sum
 * of squared distances at the assignment step.  The sums are added atomically, so two runs agree
 * to rounding, not bit for bit.  Synchronous on `stream`; allocates and frees 5*n*m bytes of
 * device scratch (plus the sums).  Replaces the codebook. */
#define PSC_START_SEEDED 0
#define PSC_START_CURRENT 1
int psc_train_pq_device(psc_index *idx, const float *x_dev, int64_t n, int iters, uint64_t seed, int start,
                        double *objective_out_host, psc_stream stream);

/* Index assignment (Section 3.1 weighted distance-estimator objective, Section
 * 3.2 simulated annealing): for each sub-quantizer, anneal a bijection pi from
 * centroid numbers to 8-bit indices for n_iter iterations (start temperature
 * t0, multiplied by t_decay after every iteration, weight alpha^f(d)); a
 * proposal is accepted when it lowers the loss or, otherwise, with probability
 * equal to the temperature.  The paper's values: n_iter = 500000, t0 = 0.7,
 * t_decay = 0.9^(1/500), alpha = 0.5.  Sub-quantizer j uses seed + j; proposal
 * number it takes SplitMix64 draws 3it, 3it+1, 3it+2 of that seed.
 * The codebook rows are renumbered in place (new row pi[i] = old row i), so
 * everything downstream works with the renumbered codebook only.
 * perm_out_host (may be NULL) [m][256] receives pi; loss_out_host (may be NULL)
 * [m][2] receives the loss before and after. */
int psc_optimize_index_assignment(psc_index *idx, int64_t n_iter, double t0, double t_decay,
                                  double alpha, uint64_t seed, uint8_t *perm_out_host,
                                  double *loss_out_host);

/* The same annealing on the ranking loss of Section 3.1 ("PolyR" in Section 4.2): the loss of an
 * assignment is the sum over ordered pairs of centroids (i, j), j != i, of
 * alpha_rank(i,j) * ell_r, with alpha_r = 1/r and ell_r = 1 + 1/2 + ... + 1/r, where rank(i,j) is
 * the place of j among the centroids ordered by distance to i (the nearest other centroid has rank
 * 1) and r = the number of centroids that lie farther from i than j does, yet whose index is
 * nearer to pi[i] in Hamming distance than pi[j] is.  Same proposals, acceptance rule, random
 * draws, renumbering and outputs as psc_optimize_index_assignment; an iteration recounts all 65536
 * pairs (about 0.1 ms), so the paper's 500000 iterations take about a minute per sub-quantizer
 * (one host thread each).  A comparison baseline: the paper retains the distance-estimator loss. */
int psc_optimize_index_assignment_ranking(psc_index *idx, int64_t n_iter, double t0, double t_decay,
                                          uint64_t seed, uint8_t *perm_out_host, double *loss_out_host);

/* Install / read back the codebook, cb_host [m][256][dim/m] float32. */
int psc_set_codebook(psc_index *idx, const float *cb_host);
int psc_get_codebook(const psc_index *idx, float *cb_host);

/* ------------------------------------------------------------------ transformation in front of the quantizer */
/* Section 4.3 applies an optimized rotation before encoding with the product quantizer; the
 * additional results also reduce the dimension inside that transformation (128-D to 64-D in front
 * of 8 sub-quantizers, 96-D to 80-D in front of 20).  psc_set_rotation installs the matrix
 * r_host [dim][dim_in] (float32, row-major; dim = the index's dimension, 1 <= dim_in <= 4096; any
 * matrix: a rotation, a projection, their product) -- learning it is the caller's business.
 * psc_rotate computes y_dev [n][dim] = x_dev [n][dim_in] . r^T on the matrix cores in full float32
 * (products accumulated in ascending coordinate order): the step in front of psc_encode,
 * psc_build_lut, psc_search, psc_knn_graph, psc_ivf_assign_encode and psc_ivf_search, which all
 * take vectors of the index's own dimension.  Both buffers are the caller's. */
int psc_set_rotation(psc_index *idx, const float *r_host, int dim_in);
int psc_rotate(const psc_index *idx, const float *x_dev, int64_t n, float *y_dev, psc_stream stream);

/* Bring the index's device image up to date now (codebook; transformation matrix; coarse centroids
 * and per-list tables if an inverted file is set up), so that later device calls neither allocate nor block.
 * Synchronous. */
int psc_prepare(const psc_index *idx, psc_stream stream);

/* ------------------------------------------------------------------ device operations */
/* PQ encoding: codes_dev [n][m], byte j = nearest centroid of sub-quantizer j
 * to sub-vector j of x_dev [n][dim] (float32), lowest index on equal distance.
 * Distances are accumulated in float32, coordinates in ascending order. */
int psc_encode(const psc_index *idx, const float *x_dev, int64_t n, uint8_t *codes_dev,
               psc_stream stream);

/* ADC tables (Section 4.2 "ADC"): lut_dev [nq][m][256] float32,
 * lut[q][j][c] = squared Euclidean distance between sub-vector j of query q and
 * centroid c of sub-quantizer j.  For even dim/m the tables are computed on the matrix cores
 * (full float32 MFMA) as |q'|^2 - 2 q'.c' + |c'|^2 with both sides centred on the
 * sub-quantizer's mean centroid, clamped at 0; an entry that comes out below 1/16 of
 * |q'|^2 + |c'|^2 (the terms have cancelled: a centroid close to the query) is recomputed by
 * direct differences, so that every entry is accurate to a few 1e-6 of its own value.
 * qcodes_dev (may be NULL) [nq][m] receives the query's own code = per
 * row the index of the smallest entry of that very table (lowest on ties). */
int psc_build_lut(const psc_index *idx, const float *q_dev, int64_t nq, float *lut_dev,
                  uint8_t *qcodes_dev, psc_stream stream);

/* Hamming filter alone (Section 3.3 first step): nsurv_dev [nq] int64 receives,
 * per query, the number of codes whose Hamming distance to the query code over
 * all 8m bits is <= ht.  hdist_dev (may be NULL; small inputs) [nq][n] uint8
 * receives every distance. */
int psc_hamming_filter(int m, const uint8_t *qcodes_dev, int64_t nq, const uint8_t *codes_dev,
                       int64_t n, int ht, int64_t *nsurv_dev, uint8_t *hdist_dev,
                       psc_stream stream);

/* Adjusting the threshold (Section 4.2: thresholds are set on a training set so that the Hamming
 * comparison removes at least a given share of the points).
 * psc_hamming_histogram: hist_dev [8m+1] int64 (device; overwritten) receives, for h = 0..8m, the
 * number of (query code, code) pairs at Hamming distance exactly h, over all nq*n pairs.
 * psc_threshold_for_rate (host only, no GPU work): the largest ht such that the pairs at
 * distance <= ht are at most max_keep_fraction of all pairs of hist_host [nbits+1]; -1 if not
 * even ht = 0 keeps that few, PSC_EINVAL (-1 as well) on a null or empty histogram. */
int psc_hamming_histogram(int m, const uint8_t *qcodes_dev, int64_t nq, const uint8_t *codes_dev,
                          int64_t n, int64_t *hist_dev, psc_stream stream);
int psc_threshold_for_rate(const int64_t *hist_host, int nbits, double max_keep_fraction);

/* The fused scan (Section 3.3; Section 4.2 "dual"): for every query q and code i,
 * keep i iff hamming(qcodes[q], codes[i]) <= ht (ht >= 8m keeps everything = pure
 * ADC search); score survivors with dist = sum_j lut[q][j][codes[i][j]] (float32,
 * j ascending); return the k smallest by (dist, id) ascending, lower id first on
 * equal distance, in ids_dev [nq][k] (int64) and dists_dev [nq][k] (float32),
 * padded with id -1 / distance +inf when fewer than k survive.
 * 1 <= k <= PSC_MAX_K, ht >= 0, n < 2^40.  Workspace: psc_scan_workspace_bytes.
 * Table entries must not be negative (they are squared distances; psc_build_lut clamps at 0):
 * the scan rejects a survivor as soon as the sum over its first sub-quantizers exceeds the
 * query's current k-th best distance.
 * The Hamming test is exact on every route the library takes: xor / popcount on the vector
 * units, or (64-bit codes, 9 queries or more, selective thresholds) an int8 dot product of
 * +-1 expansions on the matrix cores, whose sign gives the same verdict.
 * psc_set_filter_route forces one of the two where both apply (process-wide; a measurement aid,
 * results do not depend on it); psc_last_scan_route names the kernel, tile shape, database
 * slices and workgroup count the calling thread's last scan launched, e.g.
 * "scan_mfma_kernel m=8 tq=16 waves=16 slices=2 tiles=738" ("" before the first scan). */
#define PSC_ROUTE_AUTO 0
#define PSC_ROUTE_POPCOUNT 1
#define PSC_ROUTE_MFMA 2
int psc_set_filter_route(int route);
const char *psc_last_scan_route(void);
size_t psc_scan_workspace_bytes(int m, int64_t nq, int64_t n, int k);
int psc_scan(int m, const float *lut_dev, const uint8_t *qcodes_dev, int64_t nq,
             const uint8_t *codes_dev, int64_t n, int ht, int k, int64_t *ids_dev,
             float *dists_dev, void *workspace_dev, size_t workspace_bytes, psc_stream stream);

/* psc_scan for callers that cannot allocate device memory or pass a workspace (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): same arguments, kernels
 * and results as psc_scan, but the scan's scratch memory (status word, shared thresholds, partial
 * result lists) is a fixed array of PSC_STATIC_SCRATCH_BYTES that the library holds in the
 * device's global memory from load time until the process ends -- one copy per GPU.  The call
 * allocates and frees nothing.  Sizes whose psc_scan_workspace_bytes exceeds the array are
 * rejected with PSC_EINVAL.  Every call on a GPU uses that GPU's one array (the call clears what
 * must start cleared): calls that overlap on one GPU -- two streams, two threads -- race; issue
 * them on one stream.  The first call on a device looks the array's address up; the HIP runtime
 * places the array in that device's memory at that moment, once per process. */
#define PSC_STATIC_SCRATCH_BYTES (32u << 20)
int psc_scan_static(int m, const float *lut_dev, const uint8_t *qcodes_dev, int64_t nq,
                    const uint8_t *codes_dev, int64_t n, int ht, int k, int64_t *ids_dev,
                    float *dists_dev, psc_stream stream);

/* Whole flat search from raw queries q_dev [nq][dim]: psc_build_lut + psc_scan,
 * tables and query codes living in the workspace (psc_search_workspace_bytes). */
size_t psc_search_workspace_bytes(const psc_index *idx, int64_t nq, int64_t n, int k);
int psc_search(const psc_index *idx, const float *q_dev, int64_t nq, const uint8_t *codes_dev,
               int64_t n, int ht, int k, int64_t *ids_dev, float *dists_dev, void *workspace_dev,
               size_t workspace_bytes, psc_stream stream);

/* k-NN graph (Section 5): for every row i of x_dev [n][dim] the k nearest other rows:
 * tables from the raw vector x_i, bit string = its stored code codes_dev[i], database = all n
 * codes, row i itself never returned (rows with identical codes but another number stay
 * eligible).  Same filter, scoring, order and padding as psc_scan; ids_dev / dists_dev [n][k].
 * Queries are processed in chunks of 32768.  Workspace: psc_knn_graph_workspace_bytes. */
size_t psc_knn_graph_workspace_bytes(const psc_index *idx, int64_t n, int k);
int psc_knn_graph(const psc_index *idx, const float *x_dev, const uint8_t *codes_dev, int64_t n,
                  int ht, int k, int64_t *ids_dev, float *dists_dev, void *workspace_dev,
                  size_t workspace_bytes, psc_stream stream);

/* ------------------------------------------------------------------ inverted file with residual codes (Section 4.3) */
/* Coarse quantizer: nlist (<= 16384) centroids of dim floats (dim % 4 == 0, dim <= 1024).
 * psc_ivf_train_coarse runs k-means on x_host [n][dim] (assignment step on the current
 * device, synchronous, allocates and frees its own scratch); psc_ivf_set_coarse installs
 * given centroids.  Either call forgets previously set lists. */
int psc_ivf_train_coarse(psc_index *idx, const float *x_host, int64_t n, int nlist, int iters, uint64_t seed);
int psc_ivf_set_coarse(psc_index *idx, const float *centroids_host, int nlist);
/* psc_ivf_train_coarse with the training vectors already in device memory (x_dev [n][dim],
 * n < 2^31) and the whole iteration on the device: same seeded start, assignment by the
 * nearest-centroid kernel, sums in double precision (atomic adds: runs agree to rounding), an
 * empty cell restarts on the lowest-numbered member of the most populated cell.  Synchronous on
 * `stream`; allocates and frees its scratch. */
int psc_ivf_train_coarse_device(psc_index *idx, const float *x_dev, int64_t n, int nlist, int iters,
                                uint64_t seed, psc_stream stream);
int psc_ivf_get_coarse(const psc_index *idx, float *centroids_host);

/* Index construction: list_no_dev [n] (int32) = nearest coarse centroid of each row of
 * x_dev [n][dim] (squared L2 in float32, lowest number on ties); rescodes_dev (may be NULL)
 * [n][m] = PQ code of the residual x - centroid[list_no]. */
int psc_ivf_assign_encode(const psc_index *idx, const float *x_dev, int64_t n, int32_t *list_no_dev,
                          uint8_t *rescodes_dev, psc_stream stream);

/* The inverted lists, borrowed (the caller keeps them alive and unchanged while searching):
 * codes_dev [n][m] residual codes grouped by list, ids_dev [n] (int32, >= 0) the id of each
 * stored code, offsets_dev [nlist+1] (int64, device memory) list l = rows offsets[l] ..
 * offsets[l+1]-1.  codes_dev must be 16-byte aligned.  The call copies the offsets to the host
 * once (synchronously) to check them (0 first, n last, never decreasing) and to note the longest
 * list, which decides which scan kernels can serve the index.  No list may hold more than 2^27
 * codes (PSC_EINVAL): the scan addresses a code by its position inside its list. */
int psc_ivf_set_lists(psc_index *idx, const int64_t *offsets_dev, const uint8_t *codes_dev,
                      const int32_t *ids_dev, int64_t n);

/* Search: for every query the nprobe nearest coarse centroids (squared L2 in float32, lower list
 * number on ties; nprobe is clipped to nlist, at most 1024); for every probed list l the
 * residual q - centroid[l] gives that list's ADC tables and the query's bit string for that
 * list; the list's codes are filtered (Hamming <= ht) and scored as in psc_scan; one ranking by
 * (distance, id) over the union of the probed lists, ids taken from ids_dev.  No cap on lists
 * or distance evaluations.  Both exact forms of the Hamming test of psc_scan exist here too (the
 * matrix-core one is taken for 64-bit codes, thresholds up to 17 and a dozen or more (query,
 * list) pairs per list; psc_set_filter_route overrides as for psc_scan).
 * probed_out_dev (may be NULL) [nq][nprobe] int32 receives the probed lists in ascending
 * coarse distance; qcodes_out_dev (may be NULL) [nq][nprobe][m] the per-list query codes.
 * The tables are normally not stored per (query, list): with o the mean coarse centroid they split
 * into ||c||^2 - 2 (q-o)_j . c (one table per query), 2 (centroid[l]-o)_j . c (one per list) and
 * the number ||(q-centroid[l])_j||^2 per (query, list, j), which are added up as a list is scanned;
 * the bit string is the arg-min of the summed float32 rows, lowest index on ties.  The two cross
 * terms are larger than the entries they add up to by about rho = 2 |centroid[l]-o|_j /
 * (sqrt(dim/m) x rms norm of the centroids of sub-quantizer j); an index whose largest rho exceeds
 * 16 (coarse centroids spread very far apart compared with the residuals) would lose too many
 * bits, so for such an index every (query, list) table is built by direct differences and stored
 * (slower; nq*nprobe*m KiB more workspace) -- psc_last_scan_route then ends in "+direct-tables".
 * The per-list tables (nlist*m KiB) belong to the index's device image and are rebuilt by the
 * first search after the codebook or the coarse centroids changed (that call blocks; see
 * psc_prepare).
 * Up to 4096 (query, list) pairs are scanned one per workgroup in order of coarse rank (low
 * latency for a few queries); larger batches are grouped by list so that up to 16 queries share
 * every code load.
 * The workspace (psc_ivf_search_workspace_bytes: coarse distances nq*nlist*4 bytes, the
 * queries' tables nq*m KiB, and nq*nprobe*(12 k + 24) bytes of jobs and partial lists) starts
 * with the status word psc_workspace_status reads. */
size_t psc_ivf_search_workspace_bytes(const psc_index *idx, int64_t nq, int nprobe, int k);
int psc_ivf_search(const psc_index *idx, const float *q_dev, int64_t nq, int nprobe, int ht, int k,
                   int64_t *ids_dev, float *dists_dev, int32_t *probed_out_dev, uint8_t *qcodes_out_dev,
                   void *workspace_dev, size_t workspace_bytes, psc_stream stream);

/* ------------------------------------------------------------------ inverted multi-index (Section 4.3, Table 2) */
/* The coarse level is a product quantizer: the first dim/2 coordinates are quantized with k1
 * centroids c1_host [k1][dim/2], the others with k2 centroids c2_host [k2][dim/2] (k1, k2 <= 16384,
 * k1*k2 < 2^31; dim % 8 == 0, m even), which gives k1*k2 cells; cell (a, b) has number a*k2 + b and
 * centroid (c1[a], c2[b]).  Training the two halves is two plain coarse trainings in dimension
 * dim/2 (psc_ivf_train_coarse* on an index of that dimension).  The call forgets earlier cell lists. */
int psc_imi_set_coarse(psc_index *idx, const float *c1_host, int k1, const float *c2_host, int k2);

/* Index construction: cell_no_dev [n] (int32) = the cell of each row of x_dev [n][dim] (per half the
 * nearest centroid, squared L2 in float32, lowest number on ties); rescodes_dev (may be NULL)
 * [n][m] = PQ code of the residual x - cell centroid.  Rows are processed 2^20 at a time through
 * the workspace (psc_imi_assign_workspace_bytes). */
size_t psc_imi_assign_workspace_bytes(const psc_index *idx, int64_t n);
int psc_imi_assign_encode(const psc_index *idx, const float *x_dev, int64_t n, int32_t *cell_no_dev,
                          uint8_t *rescodes_dev, void *workspace_dev, size_t workspace_bytes, psc_stream stream);

/* The cells' lists, borrowed like the lists of psc_ivf_set_lists: offsets_dev [k1*k2+1] (int64,
 * device memory; copied to the host once to be checked), codes_dev [n][m] grouped by cell (16-byte
 * aligned), ids_dev [n] (int32, >= 0). */
int psc_imi_set_lists(psc_index *idx, const int64_t *offsets_dev, const uint8_t *codes_dev, const int32_t *ids_dev,
                      int64_t n);

/* Search: every query takes cells in non-decreasing order of its squared distance to the cell
 * centroid, d1[a] + d2[b] (float32; lower cell number first on equal sums), until max_lists cells
 * (1 .. 1024) are taken or the cells taken hold max_codes codes or more (max_codes <= 0: no such
 * cap; the cell that reaches it is scanned whole; empty cells count as taken) -- the two caps of
 * Table 2.  Inside a cell: bit string and ADC tables from the residual q - cell centroid, codes
 * filtered (Hamming <= ht) and scored as in psc_scan; one ranking by (distance, id) over all cells
 * taken.  cells_out_dev (may be NULL) [nq][max_lists] int32 receives the cells taken, in order,
 * padded with -1; qcodes_out_dev (may be NULL) [nq][max_lists][m] the bit strings of those cells.
 * Cells of a multi-index hold a handful of codes each and queries rarely share one, so nothing is
 * grouped by cell: in a batch one workgroup serves one query from its first cell to its last; up
 * to 256 queries have their cells dealt out to several workgroups each (32 for a single query),
 * whose lists are merged.  The order of the cells is found in passes over the first 64, 256 and
 * max_lists cells; a pass settles the queries whose cap on codes is reached within its cells.
 * The tables are put together per cell from the query's share, the two half-centroids'
 * shares (k1 + k2 half tables, part of the index's device image as for psc_ivf_search) and
 * ||(q - cell centroid)_j||^2, or by direct differences under the rule stated at psc_ivf_search
 * (psc_last_scan_route then starts with "imi_scan_kernel+direct-tables"). */
size_t psc_imi_search_workspace_bytes(const psc_index *idx, int64_t nq, int max_lists);
int psc_imi_search(const psc_index *idx, const float *q_dev, int64_t nq, int max_lists, int64_t max_codes, int ht,
                   int k, int64_t *ids_dev, float *dists_dev, int32_t *cells_out_dev, uint8_t *qcodes_out_dev,
                   void *workspace_dev, size_t workspace_bytes, psc_stream stream);

/* Synchronise `stream` and report whether any scan that used this workspace since
 * the last call gave up on an internal wait (never expected; results of such a
 * scan are marked with id -2).  Returns 0 if clean, PSC_EHIP otherwise. */
int psc_workspace_status(void *workspace_dev, psc_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* PSC_H */
