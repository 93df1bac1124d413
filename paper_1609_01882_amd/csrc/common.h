// Internal declarations shared by the translation units of libpsc (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <mutex>
#include <vector>

#include "psc.h"

namespace psc {

void set_error(const char *fmt, ...) __attribute__((format(printf, 1, 2)));

#define PSC_HIP_TRY(expr)                                                                    \
    do {                                                                                     \
        hipError_t e_ = (expr);                                                              \
        if (e_ != hipSuccess) {                                                              \
            ::psc::set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, \
                             __LINE__);                                                      \
            return PSC_EHIP;                                                                 \
        }                                                                                    \
    } while (0)

#define PSC_REQUIRE(cond, ...)          \
    do {                                \
        if (!(cond)) {                  \
            ::psc::set_error(__VA_ARGS__); \
            return PSC_EINVAL;          \
        }                               \
    } while (0)

constexpr int kCentroids = 256;  // centroids per sub-quantizer: one byte per index

// ---- host-side training (host_train.cpp)
// Lloyd k-means on x [n][d] -> cent [ncent][d].
int host_kmeans(const float *x, int64_t n, int d, int ncent, int iters, uint64_t seed, float *cent);
// The rows k-means starts from: ncent distinct row numbers out of n (n >= ncent), from the seed.
void kmeans_start_rows(int64_t n, int ncent, uint64_t seed, int64_t *rows);
// Simulated annealing of the index assignment of one sub-quantizer; cent [256][dsub].
void host_anneal(const float *cent, int dsub, int64_t n_iter, double t0, double t_decay,
                 double alpha, uint64_t seed, uint8_t *pi, double *loss_before, double *loss_after);

// The same annealing on the ranking loss (Section 3.1 "Ranking loss").
void host_anneal_ranking(const float *cent, int dsub, int64_t n_iter, double t0, double t_decay, uint64_t seed,
                         uint8_t *pi, double *loss_before, double *loss_after);

// ---- device launchers (kernels_lut.hip)
// Row selection for tables / codes built from "virtual" rows:
//   row r uses vector x[row_idx ? row_idx[r] : r] minus (sub ? sub[sub_idx[r]] : 0).
struct RowMap {
    const int32_t *row_idx = nullptr;
    const float *sub = nullptr;       // [*][dim] vectors to subtract (coarse centroids)
    const int32_t *sub_idx = nullptr; // which one, per row (none: the first, for every row)
    // k2 > 0 (inverted multi-index): sub_idx[r] = a * k2 + b and the vector to subtract is
    // (sub[a], sub_b[b]), two half-length centroids
    const float *sub_b = nullptr;
    int k2 = 0;
};
// cross: write || c ||^2 - 2 v . c instead of || v - c ||^2 (the inverted-file scan's per-query share).
int launch_lut(const float *cb_dev, int dim, int m, const float *x_dev, int64_t nrows,
               const RowMap &map, bool cross, float *lut_dev, hipStream_t s);
int launch_encode(const float *cb_dev, int dim, int m, const float *x_dev, int64_t nrows,
                  const RowMap &map, uint8_t *codes_dev, hipStream_t s);
// Tables on the matrix cores from the centred codebook cbc [m][256][dsub] and the per-sub-quantizer
// mean centroids mu [m][dsub] (entries that cancel badly are redone from the codebook cb by direct
// differences); and the arg-min of every table row (nrows_total = rows x m).
int launch_lut_mfma(const float *cb_dev, const float *cbc_dev, const float *mu_dev, int dim, int m,
                    const float *x_dev, int64_t nrows, float *lut_dev, hipStream_t s);
int launch_row_argmin(const float *lut_dev, int64_t nrows_total, uint8_t *codes_dev, hipStream_t s);

// ---- linear transformation in front of the quantizer (kernels_rotate.hip)
// y [n][dout] = x [n][din] . R^T with the matrix stored transposed and zero-padded:
// rt [din_pad][dout_pad], din_pad a multiple of 64, dout_pad of 32.
int launch_rotate(const float *x_dev, int64_t n, int din, const float *rt_dev, int din_pad, int dout, int dout_pad,
                  float *y_dev, hipStream_t s);

// ---- device launchers (kernels_scan.hip)
// Which Hamming filter the scans take where both apply: PSC_ROUTE_* of psc_set_filter_route.
extern std::atomic<int> g_filter_route;
// The kernel and tile shape the calling thread's last scan launched ("" before the first).
const char *last_scan_route();
void note_scan_route(const char *text);  // (for the searches whose kernels live in other files)
struct ScanPlan {
    int tq = 0;          // queries per workgroup tile
    int nwaves = 0;      // waves per workgroup
    int wgs_per_cu = 1;  // workgroups of this shape a compute unit holds at a time
    int kpad = 0;        // k rounded up to a multiple of 4: the stride of a list in LDS
    int nslice = 0;      // database slices (one workgroup per (query tile, slice))
    int64_t slice_len = 0;
    int64_t tiles_one = 0;  // leading query tiles that scan the whole database in one piece
    int64_t ntiles = 0;
    size_t lds_bytes = 0;
    int pub_slots = 1;      // words per query in the shared thresholds
    size_t gthr_bytes = 0;  // per-query shared thresholds
    size_t part_bytes = 0;  // partial result lists
    size_t total_bytes = 0; // whole workspace
};
// kind: which scan the plan is for (the shapes differ)
enum { kScanFused = 0, kScanDense = 1, kScanLists = 2, kScanDenseFiltered = 3, kScanFusedMfma = 4 };
int plan_scan(int m, int64_t nq, int64_t n, int k, int kind, ScanPlan *plan);
// Per query, the k best by (distance, id) of its nlists partial lists part_d / part_i [nq][nlists][k]
// (each ascending, padded with +infinity / -1) -> ids / dists [nq][k].  status: the workspace's flag
// (a scan that gave up on a wait poisons the results).
int merge_partial_lists(const float *part_d, const int64_t *part_i, int64_t nq, int nlists, int k, const int *status,
                        int64_t *ids, float *dists, hipStream_t s);
// Words per query of the thresholds the lists of one query share, given how many lists (database
// slices, probed inverted lists) a query has.
int shared_threshold_words(int64_t lists_per_query);
// Workspace that serves a flat scan whatever route (fused or dense) the threshold selects.
size_t flat_scan_workspace_bytes(int m, int64_t nq, int64_t n, int k);
// skip_first >= 0: query q never returns database row skip_first + q (k-NN-graph mode).
// clear_status: reset the workspace's status word first (false for follow-up chunks of one call).
int launch_scan(int m, const float *lut_dev, const uint8_t *qcodes_dev, int64_t nq,
                const uint8_t *codes_dev, int64_t n, int ht, int k, int64_t skip_first,
                bool clear_status, int64_t *ids_dev, float *dists_dev, void *ws, size_t ws_bytes,
                hipStream_t s);
// lut_dev: tables of the queries minus the mean coarse centroid, [nq][m][256]; list_tab_dev:
// the lists' share of the residual tables (launch_list_tables); job_qcodes_dev: out, the query
// code of every job, in job order.
int launch_ivf_scan(int m, int tq, int nwaves, int kpad, size_t lds_bytes, const float *lut_dev,
                    const float *list_tab_dev,
                    const float *queries_dev, const float *coarse_dev, int dim, int nlist,
                    uint8_t *job_qcodes_dev, const uint8_t *codes_dev, int64_t n, int ht, int k,
                    const void *tiles_dev, const int *ntiles_dev, int64_t max_tiles,
                    const int64_t *list_off_dev, const int32_t *ext_ids_dev, const int32_t *job_slot_dev,
                    const int32_t *job_q_dev, uint32_t *gthr_dev, float *part_d, int64_t *part_i, int *status,
                    int64_t nq, int nprobe, int64_t *ids_dev, float *dists_dev, bool on_matrix_cores,
                    bool one_job_per_tile, hipStream_t s);
// Whether the grouped inverted-file scan of njobs (query, list) jobs runs its Hamming test on the
// matrix cores; if so *plan receives that kernel's tile shape (16 jobs x 16 waves).
bool ivf_scan_on_matrix_cores(int m, int ht, int k, int64_t njobs, int nlist, int64_t max_list_len, ScanPlan *plan);
int launch_hamming_histogram(int m, const uint8_t *qcodes_dev, int64_t nq, const uint8_t *codes_dev,
                             int64_t n, int64_t *hist_dev, hipStream_t s);
int launch_hamming_filter(int m, const uint8_t *qcodes_dev, int64_t nq, const uint8_t *codes_dev,
                          int64_t n, int ht, int64_t *nsurv_dev, uint8_t *hdist_dev, hipStream_t s);

// ---- inverted-file helpers (kernels_ivf.hip)
// Squared distances of rows x [n][dim] to centroids [nlist][dim] -> dist [n][nlist] (float32).
int launch_coarse_distances(const float *x_dev, int64_t n, int dim, const float *cent_dev, int nlist,
                            const float *mu_dev, float *dist_dev, hipStream_t s);
// Per row the nprobe smallest of dist [n][nlist] by (distance, list number) -> probed [n][nprobe].
// settled_dev (or null): rows r with settled_dev[r] >= 0 are left out (their row of probed is not written).
int launch_select_probes(const float *dist_dev, int64_t n, int nlist, int nprobe, const int32_t *settled_dev,
                         int32_t *probed_dev, hipStream_t s);
// Nearest centroid of each row (lowest number on ties) -> assign [n] (int32).
int launch_nearest_centroid(const float *x_dev, int64_t n, int dim, const float *cent_dev, int nlist,
                            const float *mu_dev, int32_t *assign_dev, hipStream_t s);
struct IvfJobBuffers {
    int32_t *hist;       // [nblk][2 nlist]
    int32_t *list_begin; // [2 nlist + 1] first sorted job of each sort key (see launch_build_jobs)
    int32_t *tile_begin; // [2 nlist + 1] first tile of each key; tile_begin[2 nlist] = tile count
    int32_t *job_q;      // [njobs] query of the sorted job
    int32_t *job_list;   // [njobs]
    int32_t *job_slot;   // [njobs] query * nprobe + probe rank
    void *tiles;         // [max_tiles] x 16 bytes
};
// Up to this many (query, probe) jobs are not grouped by list: each is a tile of its own
// (64 probes of 100M vectors in 4096 lists, whole search, one job per tile / grouped:
//  64 queries 0.34 / 0.45 ms, 128 queries 0.53 / 0.49 ms, 256 queries 0.83 / 0.61 ms).
constexpr int64_t kDirectJobs = 4096;
// Sort the (query, probe) jobs by key (stable in query order) and cut each key's jobs into tiles
// of at most tq.  Key = list for the jobs of a query's `pilot` nearest lists, nlist + list for
// the others: the nearest lists' tiles come first.
int launch_build_jobs(const int32_t *probed_dev, int64_t nq, int nprobe, int nlist, int pilot, int tq,
                      const IvfJobBuffers &b, hipStream_t s);

// list_tab[l][j][c] = 2 (g_l - o)_j . C[j][c] for the coarse centroids g_l = rows 0..nlist-1 of
// coarse_dev and their mean o = row nlist.
int launch_list_tables(const float *cb_dev, int dim, int m, const float *coarse_dev, int nlist,
                       float *list_tab_dev, hipStream_t s);

int launch_unsort_rows(const uint8_t *src_dev, const int32_t *job_slot_dev, int64_t njobs, int row_bytes,
                       uint8_t *dst_dev, hipStream_t s);

// ---- inverted multi-index (kernels_imi.hip)
int launch_split_halves(const float *x_dev, int64_t n, int dim, float *h1_dev, float *h2_dev, hipStream_t s);
int launch_combine_cells(const int32_t *a_dev, const int32_t *b_dev, int64_t n, int k2, int32_t *cell_dev, hipStream_t s);
// Per query the cells to visit, in order, from the l1 / l2 nearest half-centroids in order (sel*,
// rows of l1 / l2 entries) and all half distances (dist*): cells [nq][lmax] (-1 padded), ncells [nq].
// One pass over the first lcur <= lmax cells of the order.  lcur < lmax: queries whose cap on codes
// is not reached within those cells get ncells = -1 and no cells; only_marked: only queries with
// ncells = -1 are worked on.
int launch_imi_cells(const int32_t *sel1_dev, const float *dist1_dev, int k1, int l1, const int32_t *sel2_dev,
                     const float *dist2_dev, int k2, int l2, int lmax, int lcur, bool only_marked, int64_t max_codes,
                     const int64_t *offsets_dev, int64_t nq, int32_t *cells_dev, int32_t *ncells_dev, int *status_dev,
                     hipStream_t s);
// `split` workgroups per query (workgroup s over the query's cells s, s + split, ...): residual
// tables, bit strings, filter, ADC, best k; split > 1: each writes a partial list (part_* [nq][split][k])
// and the lists are merged.
int launch_imi_scan(int m, const float *lut_dev, const float *tab1_dev, const float *tab2_dev, const float *cb_dev,
                    const float *queries_dev, const float *c1_dev, const float *c2_dev, int dim, int k2,
                    const int32_t *cells_dev, const int32_t *ncells_dev, int lmax, const int64_t *offsets_dev,
                    const uint8_t *codes_dev, const int32_t *ext_ids_dev, int ht, int k, bool direct, int64_t nq,
                    uint8_t *qcodes_out_dev, int64_t *ids_dev, float *dists_dev, int split, float *part_d_dev,
                    int64_t *part_i_dev, const int *status_dev, hipStream_t s);

// ---- k-means on the device (kernels_train.hip)
// One Lloyd step of all m sub-quantizers: per row and sub-quantizer the nearest centroid
// (cell [n][m]) and its squared distance (dmin [n][m]); per cell the sum of its members
// (sum [m][256][dsub], double) and their number; per sub-quantizer the sum of the distances.
int launch_pq_lloyd_step(const float *cb_dev, int dim, int m, const float *x_dev, int64_t n, uint8_t *cell_dev,
                         float *dmin_dev, double *sum_dev, uint32_t *count_dev, double *obj_dev, hipStream_t s);
// Starting centroids: sub-vector j of row rows[j][c] for every (j, c).
int launch_pq_gather_start(const float *x_dev, int dim, int m, const int64_t *rows_dev, float *cb_dev, hipStream_t s);
// The farthest member of cell `big` of sub-quantizer j becomes the only member of the empty cell c
// (sums, counts, cell and dmin follow).  Synchronizes the stream.
int launch_pq_refill(const float *x_dev, int64_t n, int dim, int m, int j, int big, int c, uint8_t *cell_dev,
                     float *dmin_dev, double *sum_dev, uint32_t *count_dev, unsigned long long *key_dev,
                     hipStream_t s);
// cent[c] = sum[c] / count[c] where count[c] > 0 (cells of d floats).
int launch_centroid_update(const double *sum_dev, const uint32_t *count_dev, int64_t ncell, int d, float *cent_dev,
                           hipStream_t s);
int launch_gather_rows(const float *x_dev, int dim, const int64_t *rows_dev, int64_t nrows, float *out_dev,
                       hipStream_t s);
// Sums and counts of the coarse cells from an assignment [n].
int launch_coarse_accumulate(const float *x_dev, int64_t n, int dim, const int32_t *assign_dev, int ncent,
                             double *sum_dev, uint32_t *count_dev, hipStream_t s);
// The lowest-numbered member of cell `big` becomes the only member of the empty cell c.
// Synchronizes the stream.
int launch_coarse_refill(const float *x_dev, int64_t n, int dim, int big, int c, int32_t *assign_dev,
                         double *sum_dev, uint32_t *count_dev, unsigned long long *key_dev, hipStream_t s);
// Row ncent of cent_dev [ncent + 1][dim] := the mean of rows 0 .. ncent-1.
int launch_mean_centroid(float *cent_dev, int ncent, int dim, hipStream_t s);

}  // namespace psc

struct psc_index {
    // guards the lazily refreshed device image below (the `mutable` members): two host threads
    // may issue their first device call on one index at the same time
    mutable std::mutex image_lock;
    int dim = 0, m = 0, dsub = 0;
    int device = 0;
    bool has_codebook = false;
    std::vector<float> cb_host;  // [m][256][dsub], the master copy
    mutable float *cb_dev = nullptr;   // [m][256][dsub], then the centred copy, then mu [m][dsub]
    mutable bool dev_current = false;  // device copy matches cb_host
    // linear transformation in front of the quantizer (psc_set_rotation): the matrix transposed and
    // zero-padded, [rot_din_pad][rot_dout_pad]; rot_din = 0: none set
    int rot_din = 0, rot_din_pad = 0, rot_dout_pad = 0;
    std::vector<float> rot_host;
    mutable float *rot_dev = nullptr;
    mutable bool rot_current = false;
    // inverted file: coarse centroids (owned) and borrowed views of the caller's lists
    int nlist = 0;
    std::vector<float> coarse_host;  // [nlist][dim]
    mutable float *coarse_dev = nullptr;
    mutable bool coarse_current = false;
    // the lists' share of the residual tables [nlist][m][256] (launch_list_tables); follows the
    // codebook and the coarse centroids
    mutable float *list_tab_dev = nullptr;
    mutable int list_tab_nlist = 0;
    mutable bool list_tab_current = false;
    mutable int direct_tables = -1;  // 1: residual tables built per (query, list) pair; -1: not decided yet
    // inverted multi-index: product coarse quantizer (owned), half tables, borrowed cell lists
    int imi_k1 = 0, imi_k2 = 0;
    std::vector<float> imi_c1_host, imi_c2_host;  // [k1][dim/2], [k2][dim/2]
    mutable float *imi_dev = nullptr;    // [k1+1][dim/2] (mean last), [k2+1][dim/2], then the two means as one [dim] vector
    mutable bool imi_current = false;
    mutable float *imi_tab_dev = nullptr;  // [k1][m/2][256] then [k2][m/2][256]
    mutable bool imi_tab_current = false;
    mutable int imi_direct = -1;
    const int64_t *imi_off_dev = nullptr;  // [k1*k2+1]
    const uint8_t *imi_codes_dev = nullptr;
    const int32_t *imi_ids_dev = nullptr;
    int64_t imi_n = 0;
    const int64_t *list_off_dev = nullptr;  // [nlist+1]
    const uint8_t *list_codes_dev = nullptr;
    const int32_t *list_ids_dev = nullptr;
    int64_t list_n = 0;
    int64_t list_max_len = 0;  // the longest list
};
