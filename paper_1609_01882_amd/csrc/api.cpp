// C ABI of libpsc: argument checking and dispatch.  See include/psc.h for the contract.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <thread>

#include "common.h"

namespace psc {

static thread_local std::string g_error;

void set_error(const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_error = buf;
}

// The host copy is the master; the device copy is refreshed lazily by the first device
// operation that needs it, so training and codebook access work without touching the GPU.
static int mark_codebook_changed(psc_index *idx)
{
    idx->has_codebook = true;
    idx->dev_current = false;
    idx->list_tab_current = false;
    idx->direct_tables = -1;
    idx->imi_tab_current = false;
    idx->imi_direct = -1;
    return PSC_OK;
}

static int sync_codebook_to_device(const psc_index *idx)
{
    std::lock_guard<std::mutex> guard(idx->image_lock);
    if (idx->dev_current) return PSC_OK;
    // device image: the codebook, the codebook centred on each sub-quantizer's mean centroid,
    // and those means (the last two feed the matrix-core table kernel)
    const size_t n = idx->cb_host.size(), sq = (size_t)kCentroids * idx->dsub;
    std::vector<float> img(2 * n + (size_t)idx->m * idx->dsub);
    std::memcpy(img.data(), idx->cb_host.data(), n * sizeof(float));
    for (int j = 0; j < idx->m; ++j) {
        float *mu = &img[2 * n + (size_t)j * idx->dsub];
        for (int t = 0; t < idx->dsub; ++t) {
            double acc = 0.0;
            for (int c = 0; c < kCentroids; ++c) acc += idx->cb_host[j * sq + (size_t)c * idx->dsub + t];
            mu[t] = (float)(acc / kCentroids);
        }
        for (int c = 0; c < kCentroids; ++c)
            for (int t = 0; t < idx->dsub; ++t)
                img[n + j * sq + (size_t)c * idx->dsub + t] = idx->cb_host[j * sq + (size_t)c * idx->dsub + t] - mu[t];
    }
    if (!idx->cb_dev) PSC_HIP_TRY(hipMalloc((void **)&idx->cb_dev, img.size() * sizeof(float)));
    else PSC_HIP_TRY(hipDeviceSynchronize());  // kernels enqueued earlier on any stream may still read the old image
    PSC_HIP_TRY(hipMemcpy(idx->cb_dev, img.data(), img.size() * sizeof(float), hipMemcpyHostToDevice));
    idx->dev_current = true;
    return PSC_OK;
}

// Device scratch of one training call, released when the call returns.
struct DeviceScratch {
    std::vector<void *> owned;
    ~DeviceScratch()
    {
        for (void *p : owned) (void)hipFree(p);
    }
    template <class T>
    int get(T **out, size_t count)
    {
        void *p = nullptr;
        PSC_HIP_TRY(hipMalloc(&p, (count ? count : 1) * sizeof(T)));
        owned.push_back(p);
        *out = (T *)p;
        return PSC_OK;
    }
};
#define PSC_TRY(expr)                \
    do {                             \
        int rc_ = (expr);            \
        if (rc_ != PSC_OK) return rc_; \
    } while (0)

}  // namespace psc

using namespace psc;

extern "C" {

int psc_version(void) { return 100; }

const char *psc_last_error(void) { return g_error.c_str(); }

int psc_set_filter_route(int route)
{
    PSC_REQUIRE(route == PSC_ROUTE_AUTO || route == PSC_ROUTE_POPCOUNT || route == PSC_ROUTE_MFMA,
                "route must be PSC_ROUTE_AUTO, PSC_ROUTE_POPCOUNT or PSC_ROUTE_MFMA");
    g_filter_route.store(route, std::memory_order_relaxed);
    return PSC_OK;
}

const char *psc_last_scan_route(void) { return last_scan_route(); }

int psc_create(psc_index **out, int dim, int m)
{
    PSC_REQUIRE(out != nullptr, "null output pointer");
    *out = nullptr;
    PSC_REQUIRE(m == 8 || m == 16, "m must be 8 or 16, got %d", m);
    PSC_REQUIRE(dim > 0 && dim % m == 0, "dim (%d) must be a positive multiple of m (%d)", dim, m);
    PSC_REQUIRE(dim / m <= 64, "sub-vector length %d too large (max 64)", dim / m);
    psc_index *idx = new (std::nothrow) psc_index();
    if (!idx) {
        set_error("out of host memory");
        return PSC_ENOMEM;
    }
    idx->dim = dim;
    idx->m = m;
    idx->dsub = dim / m;
    try {
        idx->cb_host.assign((size_t)m * kCentroids * idx->dsub, 0.f);
    } catch (const std::bad_alloc &) {
        delete idx;
        set_error("out of host memory");
        return PSC_ENOMEM;
    }
    *out = idx;
    return PSC_OK;
}

void psc_destroy(psc_index *idx)
{
    if (!idx) return;
    if (idx->cb_dev) (void)hipFree(idx->cb_dev);
    if (idx->coarse_dev) (void)hipFree(idx->coarse_dev);
    if (idx->list_tab_dev) (void)hipFree(idx->list_tab_dev);
    if (idx->rot_dev) (void)hipFree(idx->rot_dev);
    if (idx->imi_dev) (void)hipFree(idx->imi_dev);
    if (idx->imi_tab_dev) (void)hipFree(idx->imi_tab_dev);
    delete idx;
}

int psc_train_pq(psc_index *idx, const float *x_host, int64_t n, int iters, uint64_t seed)
{
    PSC_REQUIRE(idx && x_host, "null pointer");
    PSC_REQUIRE(n >= kCentroids, "need at least 256 training vectors, got %lld", (long long)n);
    PSC_REQUIRE(iters >= 1, "iters must be >= 1");
    try {
        std::vector<float> sub((size_t)n * idx->dsub);
        for (int j = 0; j < idx->m; ++j) {
            for (int64_t i = 0; i < n; ++i)
                std::memcpy(&sub[(size_t)i * idx->dsub], x_host + (size_t)i * idx->dim + (size_t)j * idx->dsub,
                            sizeof(float) * idx->dsub);
            int rc = host_kmeans(sub.data(), n, idx->dsub, kCentroids, iters, seed + (uint64_t)j,
                                 &idx->cb_host[(size_t)j * kCentroids * idx->dsub]);
            if (rc != PSC_OK) return rc;
        }
    } catch (const std::bad_alloc &) {
        set_error("out of host memory");
        return PSC_ENOMEM;
    }
    return mark_codebook_changed(idx);
}

static int optimize_assignment(psc_index *idx, bool ranking, int64_t n_iter, double t0, double t_decay, double alpha,
                               uint64_t seed, uint8_t *perm_out_host, double *loss_out_host);

int psc_optimize_index_assignment(psc_index *idx, int64_t n_iter, double t0, double t_decay,
                                  double alpha, uint64_t seed, uint8_t *perm_out_host,
                                  double *loss_out_host)
{
    return optimize_assignment(idx, false, n_iter, t0, t_decay, alpha, seed, perm_out_host, loss_out_host);
}

int psc_optimize_index_assignment_ranking(psc_index *idx, int64_t n_iter, double t0, double t_decay, uint64_t seed,
                                          uint8_t *perm_out_host, double *loss_out_host)
{
    return optimize_assignment(idx, true, n_iter, t0, t_decay, 0.5, seed, perm_out_host, loss_out_host);
}

static int optimize_assignment(psc_index *idx, bool ranking, int64_t n_iter, double t0, double t_decay, double alpha,
                               uint64_t seed, uint8_t *perm_out_host, double *loss_out_host)
{
    PSC_REQUIRE(idx != nullptr, "null index");
    if (!idx->has_codebook) {
        set_error("no codebook: call psc_train_pq or psc_set_codebook first");
        return PSC_ESTATE;
    }
    PSC_REQUIRE(n_iter >= 0 && t0 >= 0.0 && t_decay > 0.0 && t_decay <= 1.0 && alpha > 0.0,
                "bad annealing parameters");
    const size_t sq = (size_t)kCentroids * idx->dsub;
    // sub-quantizers are independent problems (Section 3, opening): one host thread each
    std::vector<std::thread> pool;
    for (int j = 0; j < idx->m; ++j) {
        pool.emplace_back([=] {
            float *cent = &idx->cb_host[(size_t)j * sq];
            std::vector<float> renum(sq);
            uint8_t pi[kCentroids];
            double before = 0.0, after = 0.0;
            if (ranking)
                host_anneal_ranking(cent, idx->dsub, n_iter, t0, t_decay, seed + (uint64_t)j, pi, &before, &after);
            else
                host_anneal(cent, idx->dsub, n_iter, t0, t_decay, alpha, seed + (uint64_t)j, pi, &before, &after);
            for (int i = 0; i < kCentroids; ++i)
                std::memcpy(&renum[(size_t)pi[i] * idx->dsub], cent + (size_t)i * idx->dsub,
                            sizeof(float) * idx->dsub);
            std::memcpy(cent, renum.data(), sizeof(float) * sq);
            if (perm_out_host) std::memcpy(perm_out_host + (size_t)j * kCentroids, pi, kCentroids);
            if (loss_out_host) {
                loss_out_host[2 * j] = before;
                loss_out_host[2 * j + 1] = after;
            }
        });
    }
    for (auto &t : pool) t.join();
    return mark_codebook_changed(idx);
}

int psc_set_codebook(psc_index *idx, const float *cb_host)
{
    PSC_REQUIRE(idx && cb_host, "null pointer");
    std::memcpy(idx->cb_host.data(), cb_host, idx->cb_host.size() * sizeof(float));
    return mark_codebook_changed(idx);
}

int psc_get_codebook(const psc_index *idx, float *cb_host)
{
    PSC_REQUIRE(idx && cb_host, "null pointer");
    if (!idx->has_codebook) {
        set_error("no codebook");
        return PSC_ESTATE;
    }
    std::memcpy(cb_host, idx->cb_host.data(), idx->cb_host.size() * sizeof(float));
    return PSC_OK;
}

static int need_codebook(const psc_index *idx)
{
    PSC_REQUIRE(idx != nullptr, "null index");
    if (!idx->has_codebook) {
        set_error("no codebook: call psc_train_pq or psc_set_codebook first");
        return PSC_ESTATE;
    }
    return sync_codebook_to_device(idx);
}

int psc_encode(const psc_index *idx, const float *x_dev, int64_t n, uint8_t *codes_dev, psc_stream stream)
{
    int rc = need_codebook(idx);
    if (rc != PSC_OK) return rc;
    PSC_REQUIRE(n >= 0, "negative n");
    if (n == 0) return PSC_OK;
    PSC_REQUIRE(x_dev && codes_dev, "null pointer");
    return launch_encode(idx->cb_dev, idx->dim, idx->m, x_dev, n, RowMap{}, codes_dev, (hipStream_t)stream);
}

int psc_build_lut(const psc_index *idx, const float *q_dev, int64_t nq, float *lut_dev,
                  uint8_t *qcodes_dev, psc_stream stream)
{
    int rc = need_codebook(idx);
    if (rc != PSC_OK) return rc;
    PSC_REQUIRE(nq >= 0, "negative nq");
    if (nq == 0) return PSC_OK;
    PSC_REQUIRE(q_dev && lut_dev, "null pointer");
    if (idx->dsub % 2 == 0) {
        // the dense contraction of the path: matrix cores
        const size_t n = idx->cb_host.size();
        rc = launch_lut_mfma(idx->cb_dev, idx->cb_dev + n, idx->cb_dev + 2 * n, idx->dim, idx->m, q_dev, nq, lut_dev,
                             (hipStream_t)stream);
    } else {
        rc = launch_lut(idx->cb_dev, idx->dim, idx->m, q_dev, nq, RowMap{}, false, lut_dev, (hipStream_t)stream);
    }
    if (rc != PSC_OK) return rc;
    if (qcodes_dev) rc = launch_row_argmin(lut_dev, nq * idx->m, qcodes_dev, (hipStream_t)stream);
    return rc;
}

int psc_hamming_histogram(int m, const uint8_t *qcodes_dev, int64_t nq, const uint8_t *codes_dev,
                          int64_t n, int64_t *hist_dev, psc_stream stream)
{
    return launch_hamming_histogram(m, qcodes_dev, nq, codes_dev, n, hist_dev, (hipStream_t)stream);
}

int psc_threshold_for_rate(const int64_t *hist_host, int nbits, double max_keep_fraction)
{
    if (!hist_host || nbits < 1) {
        set_error("null or empty histogram");
        return PSC_EINVAL;
    }
    double total = 0.0;
    for (int h = 0; h <= nbits; ++h) total += (double)hist_host[h];
    if (total <= 0.0) {
        set_error("empty histogram");
        return PSC_EINVAL;
    }
    // largest ht with (pairs at distance <= ht) <= max_keep_fraction * total
    double kept = 0.0;
    int ht = -1;
    for (int h = 0; h <= nbits; ++h) {
        kept += (double)hist_host[h];
        if (kept <= max_keep_fraction * total) ht = h;
        else break;
    }
    return ht;
}

int psc_hamming_filter(int m, const uint8_t *qcodes_dev, int64_t nq, const uint8_t *codes_dev,
                       int64_t n, int ht, int64_t *nsurv_dev, uint8_t *hdist_dev, psc_stream stream)
{
    return launch_hamming_filter(m, qcodes_dev, nq, codes_dev, n, ht, nsurv_dev, hdist_dev, (hipStream_t)stream);
}

size_t psc_scan_workspace_bytes(int m, int64_t nq, int64_t n, int k)
{
    return flat_scan_workspace_bytes(m, nq, n, k);
}

int psc_scan(int m, const float *lut_dev, const uint8_t *qcodes_dev, int64_t nq,
             const uint8_t *codes_dev, int64_t n, int ht, int k, int64_t *ids_dev,
             float *dists_dev, void *workspace_dev, size_t workspace_bytes, psc_stream stream)
{
    return launch_scan(m, lut_dev, qcodes_dev, nq, codes_dev, n, ht, k, -1, true, ids_dev, dists_dev,
                       workspace_dev, workspace_bytes, (hipStream_t)stream);
}

}  // extern "C"

// ---------------------------------------------------------------------------------------------
// psc_scan without a caller's workspace and without any allocation: the scan's scratch memory is
// a fixed array in the device's global memory.  In host code the array's name stands for the
// symbol, not for a device address: the address is looked up once per device and only that
// pointer is handed to kernels.
// ---------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[PSC_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_lock;
void *g_scratch_ptr[kMaxDevices] = {};  // per device: where that device's copy of `scratch` lives

int static_scratch(void **out)
{
    int dev = -1;
    PSC_HIP_TRY(hipGetDevice(&dev));
    PSC_REQUIRE(dev >= 0 && dev < kMaxDevices, "device ordinal %d out of range", dev);
    std::lock_guard<std::mutex> guard(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        PSC_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        PSC_REQUIRE(p != nullptr && ((uintptr_t)p & 255) == 0, "static scratch array has no usable device address");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return PSC_OK;
}
}  // namespace

extern "C" {

int psc_scan_static(int m, const float *lut_dev, const uint8_t *qcodes_dev, int64_t nq,
                    const uint8_t *codes_dev, int64_t n, int ht, int k, int64_t *ids_dev,
                    float *dists_dev, psc_stream stream)
{
    const size_t need = flat_scan_workspace_bytes(m, nq, n, k);
    PSC_REQUIRE(need != 0, "%s", psc_last_error());
    PSC_REQUIRE(need <= (size_t)PSC_STATIC_SCRATCH_BYTES,
                "this scan needs %zu bytes of scratch memory, the static array holds %u: use psc_scan with a workspace",
                need, (unsigned)PSC_STATIC_SCRATCH_BYTES);
    void *ws = nullptr;
    int rc = static_scratch(&ws);
    if (rc != PSC_OK) return rc;
    // (launch_scan clears the status word and the shared thresholds with a small kernel, and the
    //  scan kernels write every partial list they later merge: nothing of the previous call is read)
    return launch_scan(m, lut_dev, qcodes_dev, nq, codes_dev, n, ht, k, -1, true, ids_dev, dists_dev, ws,
                       (size_t)PSC_STATIC_SCRATCH_BYTES, (hipStream_t)stream);
}

static size_t round256(size_t v) { return (v + 255) / 256 * 256; }

size_t psc_search_workspace_bytes(const psc_index *idx, int64_t nq, int64_t n, int k)
{
    if (!idx) return 0;
    const size_t scan_bytes = flat_scan_workspace_bytes(idx->m, nq, n, k);
    if (scan_bytes == 0) return 0;
    return round256(scan_bytes) + round256((size_t)nq * idx->m * kCentroids * sizeof(float)) +
           round256((size_t)nq * idx->m);
}

int psc_search(const psc_index *idx, const float *q_dev, int64_t nq, const uint8_t *codes_dev,
               int64_t n, int ht, int k, int64_t *ids_dev, float *dists_dev, void *workspace_dev,
               size_t workspace_bytes, psc_stream stream)
{
    int rc = need_codebook(idx);
    if (rc != PSC_OK) return rc;
    const size_t need = psc_search_workspace_bytes(idx, nq, n, k);
    PSC_REQUIRE(need != 0, "%s", psc_last_error());
    if (nq == 0) return PSC_OK;
    PSC_REQUIRE(workspace_dev && workspace_bytes >= need, "workspace too small: need %zu bytes, got %zu",
                need, workspace_bytes);
    PSC_REQUIRE(((uintptr_t)workspace_dev & 255) == 0, "workspace must be 256-byte aligned");
    // layout: [scan workspace (status word first)] [tables] [query codes]
    const size_t scan_bytes = round256(flat_scan_workspace_bytes(idx->m, nq, n, k));
    char *w = (char *)workspace_dev + scan_bytes;
    float *lut = (float *)w;
    w += round256((size_t)nq * idx->m * kCentroids * sizeof(float));
    uint8_t *qcodes = (uint8_t *)w;
    rc = psc_build_lut(idx, q_dev, nq, lut, qcodes, stream);
    if (rc != PSC_OK) return rc;
    return launch_scan(idx->m, lut, qcodes, nq, codes_dev, n, ht, k, -1, true, ids_dev, dists_dev,
                       workspace_dev, scan_bytes, (hipStream_t)stream);
}

// ---------------------------------------------------------------------------------------------
// k-NN graph (Section 5): every database vector in turn is the query.  Queries are processed in
// chunks so that one chunk's tables fit the workspace; each chunk is a flat scan whose query
// codes are the stored codes of the chunk's rows and which never returns a row to itself.
// ---------------------------------------------------------------------------------------------
static const int64_t kGraphChunk = 32768;
// Inverted file: the jobs of this many nearest lists of every query are scanned ahead of the rest.
// (100M vectors, 4096 lists, 64 probes, k=100: 17.8 ms with none, 15.4 with 2, 15.9 with 16.)
static const int kPilotProbes = 2;

// Scan workspace that serves both the full chunks and the shorter last chunk (whose plan may
// cut the database into more slices).
static size_t graph_scan_workspace(const psc_index *idx, int64_t n, int k)
{
    const int64_t qc = n < kGraphChunk ? n : kGraphChunk;
    const int64_t tail = n % kGraphChunk;
    size_t bytes = flat_scan_workspace_bytes(idx->m, qc, n, k);
    if (bytes == 0) return 0;
    if (n > kGraphChunk && tail != 0) {
        const size_t tb = flat_scan_workspace_bytes(idx->m, tail, n, k);
        if (tb == 0) return 0;
        if (tb > bytes) bytes = tb;
    }
    return round256(bytes);
}

size_t psc_knn_graph_workspace_bytes(const psc_index *idx, int64_t n, int k)
{
    if (!idx) return 0;
    const int64_t qc = n < kGraphChunk ? n : kGraphChunk;
    const size_t scan_bytes = graph_scan_workspace(idx, n, k);
    if (scan_bytes == 0) return 0;
    return scan_bytes + round256((size_t)qc * idx->m * kCentroids * sizeof(float));
}

int psc_knn_graph(const psc_index *idx, const float *x_dev, const uint8_t *codes_dev, int64_t n,
                  int ht, int k, int64_t *ids_dev, float *dists_dev, void *workspace_dev,
                  size_t workspace_bytes, psc_stream stream)
{
    int rc = need_codebook(idx);
    if (rc != PSC_OK) return rc;
    PSC_REQUIRE(n >= 0, "negative n");
    const size_t need = psc_knn_graph_workspace_bytes(idx, n, k);
    PSC_REQUIRE(need != 0, "%s", psc_last_error());
    if (n == 0) return PSC_OK;
    PSC_REQUIRE(x_dev && codes_dev && ids_dev && dists_dev, "null pointer");
    PSC_REQUIRE(workspace_dev && workspace_bytes >= need, "workspace too small: need %zu bytes, got %zu",
                need, workspace_bytes);
    PSC_REQUIRE(((uintptr_t)workspace_dev & 255) == 0, "workspace must be 256-byte aligned");
    // layout: [scan workspace for a full chunk (status word first)] [one chunk of tables]
    const size_t scan_ws_bytes = graph_scan_workspace(idx, n, k);
    char *scan_ws = (char *)workspace_dev;
    float *lut = (float *)((char *)workspace_dev + scan_ws_bytes);
    for (int64_t c0 = 0; c0 < n; c0 += kGraphChunk) {
        const int64_t qc = (n - c0) < kGraphChunk ? (n - c0) : kGraphChunk;
        if (idx->dsub % 2 == 0) {
            const size_t nc = idx->cb_host.size();
            rc = launch_lut_mfma(idx->cb_dev, idx->cb_dev + nc, idx->cb_dev + 2 * nc, idx->dim, idx->m,
                                 x_dev + (size_t)c0 * idx->dim, qc, lut, (hipStream_t)stream);
        } else {
            rc = launch_lut(idx->cb_dev, idx->dim, idx->m, x_dev + (size_t)c0 * idx->dim, qc, RowMap{}, false, lut,
                            (hipStream_t)stream);
        }
        if (rc != PSC_OK) return rc;
        rc = launch_scan(idx->m, lut, codes_dev + (size_t)c0 * idx->m, qc, codes_dev, n, ht, k, c0, c0 == 0,
                         ids_dev + (size_t)c0 * k, dists_dev + (size_t)c0 * k, scan_ws, scan_ws_bytes,
                         (hipStream_t)stream);
        if (rc != PSC_OK) return rc;
    }
    return PSC_OK;
}

// ---------------------------------------------------------------------------------------------
// Inverted file with residual codes (Section 4.3)
// ---------------------------------------------------------------------------------------------
static int sync_coarse_to_device(const psc_index *idx)
{
    std::lock_guard<std::mutex> guard(idx->image_lock);
    if (idx->coarse_current) return PSC_OK;
    // device image: the nlist centroids, then their mean (the origin the search's tables are taken from)
    const size_t dim = (size_t)idx->dim, nl = (size_t)idx->nlist;
    std::vector<float> img(idx->coarse_host);
    img.resize((nl + 1) * dim);
    for (size_t t = 0; t < dim; ++t) {
        double acc = 0.0;
        for (size_t l = 0; l < nl; ++l) acc += idx->coarse_host[l * dim + t];
        img[nl * dim + t] = (float)(acc / (double)nl);
    }
    const size_t bytes = img.size() * sizeof(float);
    if (idx->coarse_dev) {
        PSC_HIP_TRY(hipDeviceSynchronize());  // earlier kernels may still read the old centroids
        PSC_HIP_TRY(hipFree(idx->coarse_dev));
        idx->coarse_dev = nullptr;
    }
    PSC_HIP_TRY(hipMalloc((void **)&idx->coarse_dev, bytes));
    PSC_HIP_TRY(hipMemcpy(idx->coarse_dev, img.data(), bytes, hipMemcpyHostToDevice));
    idx->coarse_current = true;
    return PSC_OK;
}

// Part of the index's device image, like the codebook: built by the first search after the
// codebook or the coarse centroids changed (blocking, as their uploads are).
static int sync_list_tables(const psc_index *idx, hipStream_t s)
{
    std::lock_guard<std::mutex> guard(idx->image_lock);
    if (idx->list_tab_current) return PSC_OK;
    if (idx->list_tab_dev) PSC_HIP_TRY(hipDeviceSynchronize());  // earlier searches may still read the old tables
    if (idx->list_tab_dev && idx->list_tab_nlist != idx->nlist) {
        PSC_HIP_TRY(hipFree(idx->list_tab_dev));
        idx->list_tab_dev = nullptr;
    }
    if (!idx->list_tab_dev) {
        PSC_HIP_TRY(hipMalloc((void **)&idx->list_tab_dev, (size_t)idx->nlist * idx->m * kCentroids * sizeof(float)));
        idx->list_tab_nlist = idx->nlist;
    }
    int rc = launch_list_tables(idx->cb_dev, idx->dim, idx->m, idx->coarse_dev, idx->nlist, idx->list_tab_dev, s);
    if (rc != PSC_OK) return rc;
    PSC_HIP_TRY(hipStreamSynchronize(s));
    idx->list_tab_current = true;
    return PSC_OK;
}

// Whether the inverted-file search builds the residual tables one (query, list) pair at a time by
// direct differences instead of adding up a per-query share, a per-list share and a number.
// The shares are cross terms of the size |g~_j| |c| (g~ = coarse centroid minus the mean coarse
// centroid, c = a centroid of sub-quantizer j), rounded to float32, while the entries they add up
// to are of the size |c|^2: with rho = 2 |g~_j| / (sqrt(dsub) |c|_rms) the sum loses about
// log2(rho) bits.  Measured on the SIFT-like workloads rho is 1 to 2 (distance errors below 1e-6);
// beyond 16 the 1e-5 contract would have less than a factor 3 to spare, so from there the tables
// are built directly (slower: one table per pair is written and read).
constexpr double kDirectTablesRho = 16.0;

static bool ivf_direct_tables(const psc_index *idx)
{
    std::lock_guard<std::mutex> guard(idx->image_lock);
    if (idx->direct_tables >= 0) return idx->direct_tables != 0;
    const int dim = idx->dim, m = idx->m, dsub = idx->dsub, nl = idx->nlist;
    std::vector<double> o((size_t)dim, 0.0);
    for (int l = 0; l < nl; ++l)
        for (int t = 0; t < dim; ++t) o[(size_t)t] += idx->coarse_host[(size_t)l * dim + t];
    for (int t = 0; t < dim; ++t) o[(size_t)t] /= nl;
    double rho = 0.0;
    for (int j = 0; j < m; ++j) {
        double c2 = 0.0;
        for (int c = 0; c < kCentroids; ++c)
            for (int t = 0; t < dsub; ++t) {
                const double v = idx->cb_host[((size_t)j * kCentroids + c) * dsub + t];
                c2 += v * v;
            }
        const double crms = std::sqrt(c2 / kCentroids);
        double g2max = 0.0;
        for (int l = 0; l < nl; ++l) {
            double g2 = 0.0;
            for (int t = j * dsub; t < (j + 1) * dsub; ++t) {
                const double v = idx->coarse_host[(size_t)l * dim + t] - o[(size_t)t];
                g2 += v * v;
            }
            g2max = std::max(g2max, g2);
        }
        const double num = 2.0 * std::sqrt(g2max), den = std::sqrt((double)dsub) * crms;
        rho = std::max(rho, num <= kDirectTablesRho * den ? (den > 0.0 ? num / den : 0.0) : 2.0 * kDirectTablesRho);
    }
    idx->direct_tables = rho > kDirectTablesRho ? 1 : 0;
    return idx->direct_tables != 0;
}

static int need_coarse(const psc_index *idx)
{
    PSC_REQUIRE(idx != nullptr, "null index");
    if (idx->nlist == 0) {
        set_error("no coarse quantizer: call psc_ivf_train_coarse or psc_ivf_set_coarse first");
        return PSC_ESTATE;
    }
    return sync_coarse_to_device(idx);
}

static int sync_rotation_to_device(const psc_index *idx)
{
    std::lock_guard<std::mutex> guard(idx->image_lock);
    if (idx->rot_current) return PSC_OK;
    if (idx->rot_dev) {
        PSC_HIP_TRY(hipDeviceSynchronize());  // earlier kernels may still read the old matrix
        PSC_HIP_TRY(hipFree(idx->rot_dev));
        idx->rot_dev = nullptr;
    }
    const size_t bytes = idx->rot_host.size() * sizeof(float);
    PSC_HIP_TRY(hipMalloc((void **)&idx->rot_dev, bytes));
    PSC_HIP_TRY(hipMemcpy(idx->rot_dev, idx->rot_host.data(), bytes, hipMemcpyHostToDevice));
    idx->rot_current = true;
    return PSC_OK;
}

int psc_set_rotation(psc_index *idx, const float *r_host, int dim_in)
{
    PSC_REQUIRE(idx && r_host, "null pointer");
    PSC_REQUIRE(dim_in >= 1 && dim_in <= 4096, "input dimension must be in [1, 4096], got %d", dim_in);
    const int dout = idx->dim;
    const int din_pad = (dim_in + 63) / 64 * 64, dout_pad = (dout + 31) / 32 * 32;
    try {
        idx->rot_host.assign((size_t)din_pad * dout_pad, 0.f);
    } catch (const std::bad_alloc &) {
        set_error("out of host memory");
        return PSC_ENOMEM;
    }
    for (int c = 0; c < dout; ++c)
        for (int t = 0; t < dim_in; ++t) idx->rot_host[(size_t)t * dout_pad + c] = r_host[(size_t)c * dim_in + t];
    idx->rot_din = dim_in;
    idx->rot_din_pad = din_pad;
    idx->rot_dout_pad = dout_pad;
    idx->rot_current = false;
    return PSC_OK;
}

int psc_rotate(const psc_index *idx, const float *x_dev, int64_t n, float *y_dev, psc_stream stream)
{
    PSC_REQUIRE(idx != nullptr, "null index");
    if (idx->rot_din == 0) {
        set_error("no transformation: call psc_set_rotation first");
        return PSC_ESTATE;
    }
    PSC_REQUIRE(n >= 0, "negative n");
    if (n == 0) return PSC_OK;
    PSC_REQUIRE(x_dev && y_dev, "null pointer");
    int rc = sync_rotation_to_device(idx);
    if (rc != PSC_OK) return rc;
    return launch_rotate(x_dev, n, idx->rot_din, idx->rot_dev, idx->rot_din_pad, idx->dim, idx->rot_dout_pad, y_dev,
                         (hipStream_t)stream);
}

int psc_prepare(const psc_index *idx, psc_stream stream)
{
    int rc = need_codebook(idx);
    if (rc != PSC_OK) return rc;
    if (idx->rot_din != 0) {
        rc = sync_rotation_to_device(idx);
        if (rc != PSC_OK) return rc;
    }
    if (idx->nlist == 0) return PSC_OK;
    rc = need_coarse(idx);
    if (rc != PSC_OK) return rc;
    return ivf_direct_tables(idx) ? PSC_OK : sync_list_tables(idx, (hipStream_t)stream);
}

int psc_ivf_set_coarse(psc_index *idx, const float *centroids_host, int nlist)
{
    PSC_REQUIRE(idx && centroids_host, "null pointer");
    PSC_REQUIRE(nlist >= 1 && nlist <= 16384, "nlist must be in [1, 16384], got %d", nlist);
    PSC_REQUIRE(idx->dim % 4 == 0 && idx->dim <= 1024, "inverted file needs dim %% 4 == 0 and dim <= 1024");
    try {
        idx->coarse_host.assign(centroids_host, centroids_host + (size_t)nlist * idx->dim);
    } catch (const std::bad_alloc &) {
        set_error("out of host memory");
        return PSC_ENOMEM;
    }
    idx->nlist = nlist;
    idx->coarse_current = false;
    idx->list_tab_current = false;
    idx->direct_tables = -1;
    idx->list_off_dev = nullptr;  // lists built for another quantizer no longer apply
    idx->list_codes_dev = nullptr;
    idx->list_ids_dev = nullptr;
    idx->list_n = 0;
    return PSC_OK;
}

int psc_ivf_get_coarse(const psc_index *idx, float *centroids_host)
{
    PSC_REQUIRE(idx && centroids_host, "null pointer");
    if (idx->nlist == 0) {
        set_error("no coarse quantizer");
        return PSC_ESTATE;
    }
    std::memcpy(centroids_host, idx->coarse_host.data(), idx->coarse_host.size() * sizeof(float));
    return PSC_OK;
}

// k-means of the coarse quantizer: assignment on the device (the nearest-centroid kernel),
// centroid update on the host in double precision.
int psc_ivf_train_coarse(psc_index *idx, const float *x_host, int64_t n, int nlist, int iters, uint64_t seed)
{
    PSC_REQUIRE(idx && x_host, "null pointer");
    PSC_REQUIRE(nlist >= 1 && nlist <= 16384 && n >= nlist && iters >= 1, "bad coarse training arguments");
    PSC_REQUIRE(idx->dim % 4 == 0 && idx->dim <= 1024, "inverted file needs dim %% 4 == 0 and dim <= 1024");
    const int dim = idx->dim;
    std::vector<float> cent;
    std::vector<int32_t> assign;
    std::vector<double> sum;
    std::vector<int64_t> count;
    try {
        cent.resize((size_t)nlist * dim);
        assign.resize((size_t)n);
        sum.resize((size_t)nlist * dim);
        count.resize((size_t)nlist);
    } catch (const std::bad_alloc &) {
        set_error("out of host memory");
        return PSC_ENOMEM;
    }
    int rc = host_kmeans(x_host, n, dim, nlist, 0, seed, cent.data());  // 0 iterations: the seeded start only
    if (rc != PSC_OK) return rc;
    DeviceScratch scratch;
    float *x_dev = nullptr, *c_dev = nullptr;
    int32_t *a_dev = nullptr;
    PSC_TRY(scratch.get(&x_dev, (size_t)n * dim));
    PSC_TRY(scratch.get(&c_dev, (size_t)(nlist + 1) * dim));  // + the mean centroid
    PSC_TRY(scratch.get(&a_dev, (size_t)n));
    PSC_HIP_TRY(hipMemcpy(x_dev, x_host, (size_t)n * dim * sizeof(float), hipMemcpyHostToDevice));
    for (int it = 0; it < iters; ++it) {
        PSC_HIP_TRY(hipMemcpy(c_dev, cent.data(), cent.size() * sizeof(float), hipMemcpyHostToDevice));
        {   // the reference point of the matrix-core distance kernel
            std::vector<double> acc((size_t)dim, 0.0);
            for (int c = 0; c < nlist; ++c)
                for (int t = 0; t < dim; ++t) acc[(size_t)t] += cent[(size_t)c * dim + t];
            std::vector<float> mean((size_t)dim);
            for (int t = 0; t < dim; ++t) mean[(size_t)t] = (float)(acc[(size_t)t] / nlist);
            PSC_HIP_TRY(hipMemcpy(c_dev + (size_t)nlist * dim, mean.data(), (size_t)dim * sizeof(float), hipMemcpyHostToDevice));
        }
        PSC_TRY(launch_nearest_centroid(x_dev, n, dim, c_dev, nlist, c_dev + (size_t)nlist * dim, a_dev, nullptr));
        PSC_HIP_TRY(hipMemcpy(assign.data(), a_dev, (size_t)n * sizeof(int32_t), hipMemcpyDeviceToHost));
        std::fill(sum.begin(), sum.end(), 0.0);
        std::fill(count.begin(), count.end(), (int64_t)0);
        for (int64_t i = 0; i < n; ++i) {
            double *sp = &sum[(size_t)assign[i] * dim];
            const float *xi = x_host + (size_t)i * dim;
            for (int t = 0; t < dim; ++t) sp[t] += xi[t];
            ++count[assign[i]];
        }
        // empty cells: each restarts on the first member of the (currently) most populated cell;
        // the donor's own mean is left as computed
        std::vector<int64_t> pop(count);
        for (int c = 0; c < nlist; ++c) {
            if (pop[(size_t)c] != 0) continue;
            const int big = (int)(std::max_element(pop.begin(), pop.end()) - pop.begin());
            for (int64_t i = 0; i < n; ++i)
                if (assign[i] == big) {
                    for (int t = 0; t < dim; ++t) sum[(size_t)c * dim + t] = x_host[(size_t)i * dim + t];
                    count[(size_t)c] = 1;
                    --pop[(size_t)big];
                    pop[(size_t)c] = 1;
                    assign[i] = c;
                    break;
                }
        }
        for (int c = 0; c < nlist; ++c)
            if (count[c] > 0)
                for (int t = 0; t < dim; ++t)
                    cent[(size_t)c * dim + t] = (float)(sum[(size_t)c * dim + t] / (double)count[c]);
    }
    return psc_ivf_set_coarse(idx, cent.data(), nlist);
}

int psc_train_pq_device(psc_index *idx, const float *x_dev, int64_t n, int iters, uint64_t seed, int start,
                        double *objective_out_host, psc_stream stream)
{
    PSC_REQUIRE(idx && x_dev, "null pointer");
    PSC_REQUIRE(n >= kCentroids && n < (1LL << 31), "need 256 <= n < 2^31 training vectors, got %lld", (long long)n);
    PSC_REQUIRE(iters >= 1, "iters must be >= 1");
    PSC_REQUIRE(start == PSC_START_SEEDED || start == PSC_START_CURRENT, "start must be 0 (seeded) or 1 (current codebook)");
    if (start == PSC_START_CURRENT && !idx->has_codebook) {
        set_error("no codebook to continue from");
        return PSC_ESTATE;
    }
    const int dim = idx->dim, m = idx->m, dsub = idx->dsub;
    const size_t ncell = (size_t)m * kCentroids;
    hipStream_t s = (hipStream_t)stream;
    DeviceScratch scratch;
    float *cb = nullptr, *dmin = nullptr;
    double *sum = nullptr, *obj = nullptr;
    uint32_t *count = nullptr;
    uint8_t *cell = nullptr;
    unsigned long long *key = nullptr;
    int64_t *rows = nullptr;
    PSC_TRY(scratch.get(&cb, ncell * dsub));
    PSC_TRY(scratch.get(&sum, ncell * dsub));
    PSC_TRY(scratch.get(&count, ncell));
    PSC_TRY(scratch.get(&obj, (size_t)m));
    PSC_TRY(scratch.get(&cell, (size_t)n * m));
    PSC_TRY(scratch.get(&dmin, (size_t)n * m));
    PSC_TRY(scratch.get(&key, 1));
    PSC_TRY(scratch.get(&rows, ncell));
    std::vector<uint32_t> hcount;
    try {
        hcount.resize(ncell);
        if (start == PSC_START_SEEDED) {
            std::vector<int64_t> hrows(ncell);
            for (int j = 0; j < m; ++j) kmeans_start_rows(n, kCentroids, seed + (uint64_t)j, &hrows[(size_t)j * kCentroids]);
            PSC_HIP_TRY(hipMemcpyAsync(rows, hrows.data(), ncell * sizeof(int64_t), hipMemcpyHostToDevice, s));
            PSC_HIP_TRY(hipStreamSynchronize(s));  // hrows leaves scope
            PSC_TRY(launch_pq_gather_start(x_dev, dim, m, rows, cb, s));
        } else {
            PSC_HIP_TRY(hipMemcpyAsync(cb, idx->cb_host.data(), ncell * dsub * sizeof(float), hipMemcpyHostToDevice, s));
        }
    } catch (const std::bad_alloc &) {
        set_error("out of host memory");
        return PSC_ENOMEM;
    }
    for (int it = 0; it < iters; ++it) {
        PSC_TRY(launch_pq_lloyd_step(cb, dim, m, x_dev, n, cell, dmin, sum, count, obj, s));
        PSC_HIP_TRY(hipMemcpyAsync(hcount.data(), count, ncell * sizeof(uint32_t), hipMemcpyDeviceToHost, s));
        if (objective_out_host)
            PSC_HIP_TRY(hipMemcpyAsync(objective_out_host + (size_t)it * m, obj, (size_t)m * sizeof(double),
                                       hipMemcpyDeviceToHost, s));
        PSC_HIP_TRY(hipStreamSynchronize(s));
        for (int j = 0; j < m; ++j) {
            uint32_t *cj = &hcount[(size_t)j * kCentroids];
            for (int c = 0; c < kCentroids; ++c) {
                if (cj[c] != 0u) continue;
                // empty cell: it takes the member of the (currently) most populated cell that lies
                // farthest from that cell's centroid; the donor's own mean is left as computed
                const int big = (int)(std::max_element(cj, cj + kCentroids) - cj);
                if (cj[big] == 0u) continue;
                PSC_TRY(launch_pq_refill(x_dev, n, dim, m, j, big, c, cell, dmin, sum, count, key, s));
                --cj[big];
                cj[c] = 1u;
            }
        }
        PSC_TRY(launch_centroid_update(sum, count, (int64_t)ncell, dsub, cb, s));
    }
    PSC_HIP_TRY(hipMemcpyAsync(idx->cb_host.data(), cb, ncell * dsub * sizeof(float), hipMemcpyDeviceToHost, s));
    PSC_HIP_TRY(hipStreamSynchronize(s));
    return mark_codebook_changed(idx);
}

int psc_ivf_train_coarse_device(psc_index *idx, const float *x_dev, int64_t n, int nlist, int iters, uint64_t seed,
                                psc_stream stream)
{
    PSC_REQUIRE(idx && x_dev, "null pointer");
    PSC_REQUIRE(nlist >= 1 && nlist <= 16384 && n >= nlist && n < (1LL << 31) && iters >= 1,
                "bad coarse training arguments");
    PSC_REQUIRE(idx->dim % 4 == 0 && idx->dim <= 1024, "inverted file needs dim %% 4 == 0 and dim <= 1024");
    const int dim = idx->dim;
    hipStream_t s = (hipStream_t)stream;
    DeviceScratch scratch;
    float *cent = nullptr;
    int32_t *assign = nullptr;
    double *sum = nullptr;
    uint32_t *count = nullptr;
    unsigned long long *key = nullptr;
    int64_t *rows = nullptr;
    PSC_TRY(scratch.get(&cent, (size_t)(nlist + 1) * dim));  // + the mean centroid
    PSC_TRY(scratch.get(&assign, (size_t)n));
    PSC_TRY(scratch.get(&sum, (size_t)nlist * dim));
    PSC_TRY(scratch.get(&count, (size_t)nlist));
    PSC_TRY(scratch.get(&key, 1));
    PSC_TRY(scratch.get(&rows, (size_t)nlist));
    std::vector<uint32_t> hcount;
    std::vector<float> hcent;
    try {
        hcount.resize((size_t)nlist);
        hcent.resize((size_t)nlist * dim);
        std::vector<int64_t> hrows((size_t)nlist);
        kmeans_start_rows(n, nlist, seed, hrows.data());
        PSC_HIP_TRY(hipMemcpyAsync(rows, hrows.data(), (size_t)nlist * sizeof(int64_t), hipMemcpyHostToDevice, s));
        PSC_HIP_TRY(hipStreamSynchronize(s));
    } catch (const std::bad_alloc &) {
        set_error("out of host memory");
        return PSC_ENOMEM;
    }
    PSC_TRY(launch_gather_rows(x_dev, dim, rows, nlist, cent, s));
    for (int it = 0; it < iters; ++it) {
        PSC_TRY(launch_mean_centroid(cent, nlist, dim, s));
        PSC_TRY(launch_nearest_centroid(x_dev, n, dim, cent, nlist, cent + (size_t)nlist * dim, assign, s));
        PSC_TRY(launch_coarse_accumulate(x_dev, n, dim, assign, nlist, sum, count, s));
        PSC_HIP_TRY(hipMemcpyAsync(hcount.data(), count, (size_t)nlist * sizeof(uint32_t), hipMemcpyDeviceToHost, s));
        PSC_HIP_TRY(hipStreamSynchronize(s));
        for (int c = 0; c < nlist; ++c) {
            if (hcount[(size_t)c] != 0u) continue;
            // empty cell: restart it on the first member of the (currently) most populated cell
            const int big = (int)(std::max_element(hcount.begin(), hcount.end()) - hcount.begin());
            if (hcount[(size_t)big] == 0u) continue;
            PSC_TRY(launch_coarse_refill(x_dev, n, dim, big, c, assign, sum, count, key, s));
            --hcount[(size_t)big];
            hcount[(size_t)c] = 1u;
        }
        PSC_TRY(launch_centroid_update(sum, count, nlist, dim, cent, s));
    }
    PSC_HIP_TRY(hipMemcpyAsync(hcent.data(), cent, hcent.size() * sizeof(float), hipMemcpyDeviceToHost, s));
    PSC_HIP_TRY(hipStreamSynchronize(s));
    return psc_ivf_set_coarse(idx, hcent.data(), nlist);
}

int psc_ivf_assign_encode(const psc_index *idx, const float *x_dev, int64_t n, int32_t *list_no_dev,
                          uint8_t *rescodes_dev, psc_stream stream)
{
    int rc = need_coarse(idx);
    if (rc != PSC_OK) return rc;
    PSC_REQUIRE(n >= 0, "negative n");
    if (n == 0) return PSC_OK;
    PSC_REQUIRE(x_dev && list_no_dev, "null pointer");
    rc = launch_nearest_centroid(x_dev, n, idx->dim, idx->coarse_dev, idx->nlist,
                                 idx->coarse_dev + (size_t)idx->nlist * idx->dim, list_no_dev, (hipStream_t)stream);
    if (rc != PSC_OK || !rescodes_dev) return rc;
    rc = need_codebook(idx);
    if (rc != PSC_OK) return rc;
    RowMap map;
    map.sub = idx->coarse_dev;
    map.sub_idx = list_no_dev;
    return launch_encode(idx->cb_dev, idx->dim, idx->m, x_dev, n, map, rescodes_dev, (hipStream_t)stream);
}

int psc_ivf_set_lists(psc_index *idx, const int64_t *offsets_dev, const uint8_t *codes_dev,
                      const int32_t *ids_dev, int64_t n)
{
    PSC_REQUIRE(idx != nullptr, "null index");
    if (idx->nlist == 0) {
        set_error("no coarse quantizer");
        return PSC_ESTATE;
    }
    PSC_REQUIRE(offsets_dev && n >= 0 && (n == 0 || (codes_dev && ids_dev)), "null pointer");
    PSC_REQUIRE(((uintptr_t)codes_dev & 15) == 0, "list codes must be 16-byte aligned");
    // the longest list decides which scan kernels can serve the index: read the boundaries once
    int64_t longest = 0;
    try {
        std::vector<int64_t> off((size_t)idx->nlist + 1);
        PSC_HIP_TRY(hipMemcpy(off.data(), offsets_dev, off.size() * sizeof(int64_t), hipMemcpyDeviceToHost));
        PSC_REQUIRE(off[0] == 0 && off[(size_t)idx->nlist] == n, "list offsets must start at 0 and end at n");
        for (int l = 0; l < idx->nlist; ++l) {
            PSC_REQUIRE(off[(size_t)l + 1] >= off[(size_t)l], "list offsets must not decrease (list %d)", l);
            longest = std::max(longest, off[(size_t)l + 1] - off[(size_t)l]);
        }
    } catch (const std::bad_alloc &) {
        set_error("out of host memory");
        return PSC_ENOMEM;
    }
    PSC_REQUIRE(longest <= ((int64_t)1 << 27), "a list holds %lld codes; at most 2^27 per list", (long long)longest);
    idx->list_off_dev = offsets_dev;
    idx->list_codes_dev = codes_dev;
    idx->list_ids_dev = ids_dev;
    idx->list_n = n;
    idx->list_max_len = longest;
    return PSC_OK;
}

namespace {
struct IvfLayout {
    ScanPlan plan;
    bool direct;
    int64_t njobs, nblk, max_tiles;
    size_t off_status, off_gthr, off_dist, off_probed, off_hist, off_list_begin, off_tile_begin, off_job_q, off_job_list,
        off_job_slot, off_tiles, off_lut, off_qcodes, off_part_d, off_part_i, total;
};

int ivf_layout(const psc_index *idx, int64_t nq, int nprobe, int k, IvfLayout *L)
{
    PSC_REQUIRE(idx && idx->nlist > 0, "no coarse quantizer");
    PSC_REQUIRE(nq >= 0 && nprobe >= 1, "bad nq/nprobe");
    if (nprobe > idx->nlist) nprobe = idx->nlist;
    PSC_REQUIRE(nprobe <= 1024, "at most 1024 probes");
    L->njobs = nq * nprobe;
    PSC_REQUIRE(L->njobs < 0x7fffffffLL, "too many (query, list) jobs");
    // (few jobs are tiles of their own: the narrowest tile shape then wastes the least filter work)
    int rc = plan_scan(idx->m, L->njobs > kDirectJobs ? L->njobs : 1, idx->list_n, k, kScanLists, &L->plan);
    if (rc != PSC_OK) return rc;
    L->nblk = (nq + 15) / 16;
    L->max_tiles = L->njobs <= kDirectJobs ? L->njobs : L->njobs / L->plan.tq + 2 * (int64_t)idx->nlist;
    size_t o = 0;
    auto take = [&](size_t bytes) {
        size_t at = o;
        o += round256(bytes);
        return at;
    };
    L->off_status = take(256);
    L->off_gthr = take((size_t)nq * shared_threshold_words(nprobe) * sizeof(uint32_t));
    L->off_dist = take((size_t)nq * idx->nlist * sizeof(float));
    L->off_probed = take((size_t)L->njobs * sizeof(int32_t));
    L->off_hist = take((size_t)L->nblk * 2 * idx->nlist * sizeof(int32_t));
    L->off_list_begin = take((size_t)(2 * idx->nlist + 1) * sizeof(int32_t));
    L->off_tile_begin = take((size_t)(2 * idx->nlist + 1) * sizeof(int32_t));
    L->off_job_q = take((size_t)L->njobs * sizeof(int32_t));
    L->off_job_list = take((size_t)L->njobs * sizeof(int32_t));
    L->off_job_slot = take((size_t)L->njobs * sizeof(int32_t));
    L->off_tiles = take((size_t)L->max_tiles * 16);
    // the queries' share of the tables, or (direct tables) one table per (query, list) pair
    L->direct = idx->has_codebook && ivf_direct_tables(idx);
    L->off_lut = take((size_t)(L->direct ? L->njobs : nq) * idx->m * kCentroids * sizeof(float));
    L->off_qcodes = take((size_t)L->njobs * idx->m);
    L->off_part_d = take((size_t)L->njobs * k * sizeof(float));
    L->off_part_i = take((size_t)L->njobs * k * sizeof(int64_t));
    L->total = o;
    return PSC_OK;
}
}  // namespace

size_t psc_ivf_search_workspace_bytes(const psc_index *idx, int64_t nq, int nprobe, int k)
{
    IvfLayout L;
    if (ivf_layout(idx, nq, nprobe, k, &L) != PSC_OK) return 0;
    return L.total;
}

int psc_ivf_search(const psc_index *idx, const float *q_dev, int64_t nq, int nprobe, int ht, int k,
                   int64_t *ids_dev, float *dists_dev, int32_t *probed_out_dev, uint8_t *qcodes_out_dev,
                   void *workspace_dev, size_t workspace_bytes, psc_stream stream)
{
    int rc = need_codebook(idx);
    if (rc != PSC_OK) return rc;
    rc = need_coarse(idx);
    if (rc != PSC_OK) return rc;
    if (!idx->list_off_dev) {
        set_error("no inverted lists: call psc_ivf_set_lists first");
        return PSC_ESTATE;
    }
    PSC_REQUIRE(ht >= 0, "ht must be >= 0");
    IvfLayout L;
    rc = ivf_layout(idx, nq, nprobe, k, &L);
    if (rc != PSC_OK) return rc;
    if (nprobe > idx->nlist) nprobe = idx->nlist;
    if (nq == 0) return PSC_OK;
    PSC_REQUIRE(q_dev && ids_dev && dists_dev, "null pointer");
    PSC_REQUIRE(workspace_dev && workspace_bytes >= L.total, "workspace too small: need %zu bytes, got %zu",
                L.total, workspace_bytes);
    PSC_REQUIRE(((uintptr_t)workspace_dev & 255) == 0, "workspace must be 256-byte aligned");
    hipStream_t s = (hipStream_t)stream;
    char *w = (char *)workspace_dev;
    float *dist = (float *)(w + L.off_dist);
    int32_t *probed = (int32_t *)(w + L.off_probed);
    IvfJobBuffers jb;
    jb.hist = (int32_t *)(w + L.off_hist);
    jb.list_begin = (int32_t *)(w + L.off_list_begin);
    jb.tile_begin = (int32_t *)(w + L.off_tile_begin);
    jb.job_q = (int32_t *)(w + L.off_job_q);
    jb.job_list = (int32_t *)(w + L.off_job_list);
    jb.job_slot = (int32_t *)(w + L.off_job_slot);
    jb.tiles = w + L.off_tiles;
    float *lut = (float *)(w + L.off_lut);
    uint8_t *qcodes = (uint8_t *)(w + L.off_qcodes);

    // 1. coarse quantization of the queries and choice of the lists
    rc = launch_coarse_distances(q_dev, nq, idx->dim, idx->coarse_dev, idx->nlist,
                                 idx->coarse_dev + (size_t)idx->nlist * idx->dim, dist, s);
    if (rc != PSC_OK) return rc;
    rc = launch_select_probes(dist, nq, idx->nlist, nprobe, nullptr, probed, s);
    if (rc != PSC_OK) return rc;
    if (probed_out_dev)
        PSC_HIP_TRY(hipMemcpyAsync(probed_out_dev, probed, (size_t)L.njobs * sizeof(int32_t),
                                   hipMemcpyDeviceToDevice, s));
    // 2. jobs grouped by list, cut into tiles of the shape of the scan kernel that will run
    ScanPlan plan = L.plan;
    const bool on_matrix_cores = L.njobs > kDirectJobs &&
                                 ivf_scan_on_matrix_cores(idx->m, ht, k, L.njobs, idx->nlist, idx->list_max_len, &plan);
    rc = launch_build_jobs(probed, nq, nprobe, idx->nlist, kPilotProbes, plan.tq, jb, s);
    if (rc != PSC_OK) return rc;
    // 3. the queries' and the lists' shares of the residual tables (put together per tile by the
    //    scan, which also derives each job's query code from them)
    RowMap map;
    const float *list_tab = nullptr;
    if (L.direct) {  // one finished table per job: row = the job's query minus its list's centroid
        map.row_idx = jb.job_q;
        map.sub = idx->coarse_dev;
        map.sub_idx = jb.job_list;
        rc = launch_lut(idx->cb_dev, idx->dim, idx->m, q_dev, L.njobs, map, false, lut, s);
        if (rc != PSC_OK) return rc;
    } else {
        map.sub = idx->coarse_dev + (size_t)idx->nlist * idx->dim;  // the mean coarse centroid
        rc = launch_lut(idx->cb_dev, idx->dim, idx->m, q_dev, nq, map, true, lut, s);
        if (rc != PSC_OK) return rc;
        rc = sync_list_tables(idx, s);
        if (rc != PSC_OK) return rc;
        list_tab = idx->list_tab_dev;
    }
    // 4. the fused scan over the tiles, 5. one merge per query over its nprobe partial lists
    rc = launch_ivf_scan(idx->m, plan.tq, plan.nwaves, plan.kpad, plan.lds_bytes, lut, list_tab, q_dev, idx->coarse_dev,
                         idx->dim, idx->nlist, qcodes, idx->list_codes_dev, idx->list_n, ht, k, jb.tiles,
                         jb.tile_begin + 2 * idx->nlist, L.max_tiles, idx->list_off_dev, idx->list_ids_dev,
                         jb.job_slot, jb.job_q, (uint32_t *)(w + L.off_gthr), (float *)(w + L.off_part_d),
                         (int64_t *)(w + L.off_part_i), (int *)(w + L.off_status), nq, nprobe, ids_dev,
                         dists_dev, on_matrix_cores, L.njobs <= kDirectJobs, s);
    if (rc != PSC_OK) return rc;
    if (qcodes_out_dev) rc = launch_unsort_rows(qcodes, jb.job_slot, L.njobs, idx->m, qcodes_out_dev, s);
    return rc;
}

// ---------------------------------------------------------------------------------------------
// Inverted multi-index (Section 4.3; caption of Table 2)
// ---------------------------------------------------------------------------------------------
int psc_imi_set_coarse(psc_index *idx, const float *c1_host, int k1, const float *c2_host, int k2)
{
    PSC_REQUIRE(idx && c1_host && c2_host, "null pointer");
    PSC_REQUIRE(k1 >= 1 && k1 <= 16384 && k2 >= 1 && k2 <= 16384, "k1 and k2 must be in [1, 16384], got %d x %d", k1, k2);
    PSC_REQUIRE((int64_t)k1 * k2 < (1LL << 31), "too many cells");
    PSC_REQUIRE(idx->dim % 8 == 0 && idx->dim <= 2048, "the multi-index needs dim %% 8 == 0 and dim <= 2048");
    const size_t half = (size_t)idx->dim / 2;
    try {
        idx->imi_c1_host.assign(c1_host, c1_host + (size_t)k1 * half);
        idx->imi_c2_host.assign(c2_host, c2_host + (size_t)k2 * half);
    } catch (const std::bad_alloc &) {
        set_error("out of host memory");
        return PSC_ENOMEM;
    }
    idx->imi_k1 = k1;
    idx->imi_k2 = k2;
    idx->imi_current = false;
    idx->imi_tab_current = false;
    idx->imi_direct = -1;
    idx->imi_off_dev = nullptr;  // cells built for another quantizer no longer apply
    idx->imi_codes_dev = nullptr;
    idx->imi_ids_dev = nullptr;
    idx->imi_n = 0;
    return PSC_OK;
}

namespace {
// device image of the product coarse quantizer: [k1 + 1][half] (last row: the mean of the rows),
// [k2 + 1][half], then the two means again as one vector of dim floats
struct ImiImage {
    const float *c1, *mu1, *c2, *mu2, *origin;
};

ImiImage imi_image(const psc_index *idx)
{
    const size_t half = (size_t)idx->dim / 2, k1 = (size_t)idx->imi_k1, k2 = (size_t)idx->imi_k2;
    ImiImage im;
    im.c1 = idx->imi_dev;
    im.mu1 = im.c1 + k1 * half;
    im.c2 = im.mu1 + half;
    im.mu2 = im.c2 + k2 * half;
    im.origin = im.mu2 + half;
    return im;
}

int sync_imi_to_device(const psc_index *idx)
{
    std::lock_guard<std::mutex> guard(idx->image_lock);
    if (idx->imi_current) return PSC_OK;
    const size_t half = (size_t)idx->dim / 2, k1 = (size_t)idx->imi_k1, k2 = (size_t)idx->imi_k2;
    std::vector<float> img((k1 + 1 + k2 + 1 + 2) * half);
    auto put = [&](const std::vector<float> &src, size_t k, float *dst) {
        std::memcpy(dst, src.data(), k * half * sizeof(float));
        for (size_t t = 0; t < half; ++t) {
            double acc = 0.0;
            for (size_t c = 0; c < k; ++c) acc += src[c * half + t];
            dst[k * half + t] = (float)(acc / (double)k);
        }
    };
    put(idx->imi_c1_host, k1, img.data());
    put(idx->imi_c2_host, k2, img.data() + (k1 + 1) * half);
    std::memcpy(&img[(k1 + 1 + k2 + 1) * half], &img[k1 * half], half * sizeof(float));
    std::memcpy(&img[(k1 + 1 + k2 + 1) * half + half], &img[(k1 + 1 + k2) * half], half * sizeof(float));
    if (idx->imi_dev) {
        PSC_HIP_TRY(hipDeviceSynchronize());  // earlier kernels may still read the old centroids
        PSC_HIP_TRY(hipFree(idx->imi_dev));
        idx->imi_dev = nullptr;
    }
    PSC_HIP_TRY(hipMalloc((void **)&idx->imi_dev, img.size() * sizeof(float)));
    PSC_HIP_TRY(hipMemcpy(idx->imi_dev, img.data(), img.size() * sizeof(float), hipMemcpyHostToDevice));
    idx->imi_current = true;
    return PSC_OK;
}

// The half-centroids' shares of the residual tables (see kernels_imi.hip), rebuilt after the
// codebook or the coarse quantizer changed.
int sync_imi_tables(const psc_index *idx, hipStream_t s)
{
    std::lock_guard<std::mutex> guard(idx->image_lock);
    if (idx->imi_tab_current) return PSC_OK;
    const size_t per = (size_t)(idx->m / 2) * kCentroids;
    if (idx->imi_tab_dev) {
        PSC_HIP_TRY(hipDeviceSynchronize());
        PSC_HIP_TRY(hipFree(idx->imi_tab_dev));
        idx->imi_tab_dev = nullptr;
    }
    PSC_HIP_TRY(hipMalloc((void **)&idx->imi_tab_dev, (size_t)(idx->imi_k1 + idx->imi_k2) * per * sizeof(float)));
    const ImiImage im = imi_image(idx);
    const int half = idx->dim / 2, mh = idx->m / 2;
    int rc = launch_list_tables(idx->cb_dev, half, mh, im.c1, idx->imi_k1, idx->imi_tab_dev, s);
    if (rc != PSC_OK) return rc;
    rc = launch_list_tables(idx->cb_dev + (size_t)mh * kCentroids * idx->dsub, half, mh, im.c2, idx->imi_k2,
                            idx->imi_tab_dev + (size_t)idx->imi_k1 * per, s);
    if (rc != PSC_OK) return rc;
    PSC_HIP_TRY(hipStreamSynchronize(s));
    idx->imi_tab_current = true;
    return PSC_OK;
}

// Same rule as for the plain inverted file (kDirectTablesRho), with the half-centroids in the
// place of the coarse centroids.
bool imi_direct_tables(const psc_index *idx)
{
    std::lock_guard<std::mutex> guard(idx->image_lock);
    if (idx->imi_direct >= 0) return idx->imi_direct != 0;
    const int half = idx->dim / 2, m = idx->m, dsub = idx->dsub;
    double rho = 0.0;
    for (int j = 0; j < m; ++j) {
        double c2 = 0.0;
        for (int c = 0; c < kCentroids; ++c)
            for (int t = 0; t < dsub; ++t) {
                const double v = idx->cb_host[((size_t)j * kCentroids + c) * dsub + t];
                c2 += v * v;
            }
        const double crms = std::sqrt(c2 / kCentroids);
        const std::vector<float> &cent = j < m / 2 ? idx->imi_c1_host : idx->imi_c2_host;
        const int k = j < m / 2 ? idx->imi_k1 : idx->imi_k2;
        const int t0 = (j < m / 2 ? j : j - m / 2) * dsub;
        double g2max = 0.0;
        std::vector<double> o((size_t)dsub, 0.0);
        for (int l = 0; l < k; ++l)
            for (int t = 0; t < dsub; ++t) o[(size_t)t] += cent[(size_t)l * half + t0 + t];
        for (int t = 0; t < dsub; ++t) o[(size_t)t] /= k;
        for (int l = 0; l < k; ++l) {
            double g2 = 0.0;
            for (int t = 0; t < dsub; ++t) {
                const double v = cent[(size_t)l * half + t0 + t] - o[(size_t)t];
                g2 += v * v;
            }
            g2max = std::max(g2max, g2);
        }
        const double num = 2.0 * std::sqrt(g2max), den = std::sqrt((double)dsub) * crms;
        rho = std::max(rho, num <= kDirectTablesRho * den ? (den > 0.0 ? num / den : 0.0) : 2.0 * kDirectTablesRho);
    }
    idx->imi_direct = rho > kDirectTablesRho ? 1 : 0;
    return idx->imi_direct != 0;
}

int need_imi(const psc_index *idx)
{
    PSC_REQUIRE(idx != nullptr, "null index");
    if (idx->imi_k1 == 0) {
        set_error("no product coarse quantizer: call psc_imi_set_coarse first");
        return PSC_ESTATE;
    }
    PSC_REQUIRE(idx->m % 2 == 0, "the multi-index needs an even number of sub-quantizers");
    return sync_imi_to_device(idx);
}

constexpr int64_t kImiAssignChunk = 1 << 20;  // rows per pass of psc_imi_assign_encode
}  // namespace

size_t psc_imi_assign_workspace_bytes(const psc_index *idx, int64_t n)
{
    if (!idx || n < 0) return 0;
    const int64_t rows = std::max<int64_t>(1, std::min(n, kImiAssignChunk));
    return round256((size_t)rows * idx->dim * sizeof(float)) + 2 * round256((size_t)rows * sizeof(int32_t));
}

int psc_imi_assign_encode(const psc_index *idx, const float *x_dev, int64_t n, int32_t *cell_no_dev,
                          uint8_t *rescodes_dev, void *workspace_dev, size_t workspace_bytes, psc_stream stream)
{
    int rc = need_imi(idx);
    if (rc != PSC_OK) return rc;
    PSC_REQUIRE(n >= 0, "negative n");
    if (n == 0) return PSC_OK;
    PSC_REQUIRE(x_dev && cell_no_dev, "null pointer");
    const size_t need = psc_imi_assign_workspace_bytes(idx, n);
    PSC_REQUIRE(workspace_dev && workspace_bytes >= need, "workspace too small: need %zu bytes, got %zu", need,
                workspace_bytes);
    PSC_REQUIRE(((uintptr_t)workspace_dev & 255) == 0, "workspace must be 256-byte aligned");
    if (rescodes_dev) {
        rc = need_codebook(idx);
        if (rc != PSC_OK) return rc;
    }
    hipStream_t s = (hipStream_t)stream;
    const ImiImage im = imi_image(idx);
    const int half = idx->dim / 2;
    const int64_t rows_max = std::min(n, kImiAssignChunk);
    char *w = (char *)workspace_dev;
    float *h1 = (float *)w, *h2 = h1 + (size_t)rows_max * half;
    int32_t *a = (int32_t *)(w + round256((size_t)rows_max * idx->dim * sizeof(float)));
    int32_t *b = (int32_t *)((char *)a + round256((size_t)rows_max * sizeof(int32_t)));
    for (int64_t r0 = 0; r0 < n; r0 += kImiAssignChunk) {
        const int64_t rows = std::min(kImiAssignChunk, n - r0);
        PSC_TRY(launch_split_halves(x_dev + (size_t)r0 * idx->dim, rows, idx->dim, h1, h2, s));
        PSC_TRY(launch_nearest_centroid(h1, rows, half, im.c1, idx->imi_k1, im.mu1, a, s));
        PSC_TRY(launch_nearest_centroid(h2, rows, half, im.c2, idx->imi_k2, im.mu2, b, s));
        PSC_TRY(launch_combine_cells(a, b, rows, idx->imi_k2, cell_no_dev + r0, s));
    }
    if (!rescodes_dev) return PSC_OK;
    RowMap map;
    map.sub = im.c1;
    map.sub_b = im.c2;
    map.sub_idx = cell_no_dev;
    map.k2 = idx->imi_k2;
    return launch_encode(idx->cb_dev, idx->dim, idx->m, x_dev, n, map, rescodes_dev, s);
}

int psc_imi_set_lists(psc_index *idx, const int64_t *offsets_dev, const uint8_t *codes_dev, const int32_t *ids_dev,
                      int64_t n)
{
    PSC_REQUIRE(idx != nullptr, "null index");
    if (idx->imi_k1 == 0) {
        set_error("no product coarse quantizer");
        return PSC_ESTATE;
    }
    PSC_REQUIRE(offsets_dev && n >= 0 && (n == 0 || (codes_dev && ids_dev)), "null pointer");
    PSC_REQUIRE(((uintptr_t)codes_dev & 15) == 0, "cell codes must be 16-byte aligned");
    const size_t ncell = (size_t)idx->imi_k1 * idx->imi_k2;
    try {
        std::vector<int64_t> off(ncell + 1);
        PSC_HIP_TRY(hipMemcpy(off.data(), offsets_dev, off.size() * sizeof(int64_t), hipMemcpyDeviceToHost));
        PSC_REQUIRE(off[0] == 0 && off[ncell] == n, "cell offsets must start at 0 and end at n");
        for (size_t l = 0; l < ncell; ++l)
            PSC_REQUIRE(off[l + 1] >= off[l], "cell offsets must not decrease (cell %zu)", l);
    } catch (const std::bad_alloc &) {
        set_error("out of host memory");
        return PSC_ENOMEM;
    }
    idx->imi_off_dev = offsets_dev;
    idx->imi_codes_dev = codes_dev;
    idx->imi_ids_dev = ids_dev;
    idx->imi_n = n;
    return PSC_OK;
}

namespace {
struct ImiLayout {
    int l1, l2;
    bool direct;
    size_t off_h1, off_h2, off_d1, off_d2, off_s1, off_s2, off_cells, off_ncells, off_lut, off_part_d, off_part_i, total;
    int split;  // workgroups per query in the scan over the cells
};

// A handful of queries leave most compute units idle with one workgroup each: their cells are dealt
// out to up to 32 workgroups per query (about 512 in all), whose lists are merged.
int imi_split(int64_t nq, int max_lists)
{
    if (nq > 256 || nq < 1) return 1;
    return (int)std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>(32, max_lists), 512 / nq));
}

int imi_layout(const psc_index *idx, int64_t nq, int max_lists, ImiLayout *L)
{
    PSC_REQUIRE(idx && idx->imi_k1 > 0, "no product coarse quantizer");
    PSC_REQUIRE(nq >= 0 && max_lists >= 1 && max_lists <= 1024, "max_lists must be in [1, 1024]");
    L->l1 = std::min(max_lists, idx->imi_k1);
    L->l2 = std::min(max_lists, idx->imi_k2);
    L->direct = idx->has_codebook && imi_direct_tables(idx);
    const size_t half = (size_t)idx->dim / 2;
    size_t o = 256;  // the status word psc_workspace_status reads
    auto take = [&](size_t bytes) {
        size_t at = o;
        o += round256(bytes);
        return at;
    };
    L->off_h1 = take((size_t)nq * half * sizeof(float));
    L->off_h2 = take((size_t)nq * half * sizeof(float));
    L->off_d1 = take((size_t)nq * idx->imi_k1 * sizeof(float));
    L->off_d2 = take((size_t)nq * idx->imi_k2 * sizeof(float));
    L->off_s1 = take((size_t)nq * L->l1 * sizeof(int32_t));
    L->off_s2 = take((size_t)nq * L->l2 * sizeof(int32_t));
    L->off_cells = take((size_t)nq * max_lists * sizeof(int32_t));
    L->off_ncells = take((size_t)nq * sizeof(int32_t));
    L->off_lut = take((size_t)nq * idx->m * kCentroids * sizeof(float));
    L->split = imi_split(nq, max_lists);
    L->off_part_d = L->off_part_i = 0;
    if (L->split > 1) {  // (sized for the largest k, which the workspace query does not know)
        L->off_part_d = take((size_t)nq * L->split * PSC_MAX_K * sizeof(float));
        L->off_part_i = take((size_t)nq * L->split * PSC_MAX_K * sizeof(int64_t));
    }
    L->total = o;
    return PSC_OK;
}
}  // namespace

size_t psc_imi_search_workspace_bytes(const psc_index *idx, int64_t nq, int max_lists)
{
    ImiLayout L;
    if (imi_layout(idx, nq, max_lists, &L) != PSC_OK) return 0;
    return L.total;
}

int psc_imi_search(const psc_index *idx, const float *q_dev, int64_t nq, int max_lists, int64_t max_codes, int ht,
                   int k, int64_t *ids_dev, float *dists_dev, int32_t *cells_out_dev, uint8_t *qcodes_out_dev,
                   void *workspace_dev, size_t workspace_bytes, psc_stream stream)
{
    int rc = need_codebook(idx);
    if (rc != PSC_OK) return rc;
    rc = need_imi(idx);
    if (rc != PSC_OK) return rc;
    if (!idx->imi_off_dev) {
        set_error("no cell lists: call psc_imi_set_lists first");
        return PSC_ESTATE;
    }
    PSC_REQUIRE(ht >= 0 && k >= 1 && k <= PSC_MAX_K, "ht must be >= 0 and k in [1, %d]", PSC_MAX_K);
    ImiLayout L;
    rc = imi_layout(idx, nq, max_lists, &L);
    if (rc != PSC_OK) return rc;
    if (nq == 0) return PSC_OK;
    PSC_REQUIRE(q_dev && ids_dev && dists_dev, "null pointer");
    PSC_REQUIRE(workspace_dev && workspace_bytes >= L.total, "workspace too small: need %zu bytes, got %zu", L.total,
                workspace_bytes);
    PSC_REQUIRE(((uintptr_t)workspace_dev & 255) == 0, "workspace must be 256-byte aligned");
    hipStream_t s = (hipStream_t)stream;
    const ImiImage im = imi_image(idx);
    const int half = idx->dim / 2;
    char *w = (char *)workspace_dev;
    float *h1 = (float *)(w + L.off_h1), *h2 = (float *)(w + L.off_h2);
    float *d1 = (float *)(w + L.off_d1), *d2 = (float *)(w + L.off_d2);
    int32_t *s1 = (int32_t *)(w + L.off_s1), *s2 = (int32_t *)(w + L.off_s2);
    int32_t *cells = (int32_t *)(w + L.off_cells), *ncells = (int32_t *)(w + L.off_ncells);
    float *lut = (float *)(w + L.off_lut);
    // 1. the two halves of the coarse quantization, each with its nearest centroids in order
    PSC_TRY(launch_split_halves(q_dev, nq, idx->dim, h1, h2, s));
    PSC_TRY(launch_coarse_distances(h1, nq, half, im.c1, idx->imi_k1, im.mu1, d1, s));
    PSC_TRY(launch_coarse_distances(h2, nq, half, im.c2, idx->imi_k2, im.mu2, d2, s));
    // 2. the cells in order of d1 + d2, cut by the caps.  With a cap on codes most queries are done
    // after a few dozen cells however many are allowed: a first pass orders 64 cells (from as many
    // nearest half-centroids), a second one 256, and only the queries these do not settle go through
    // the selection of all L.l1 / L.l2 half-centroids and the full order.
    const int schedule[3] = {64, 256, max_lists};
    bool marked = false;  // a pass before this one has left queries marked (ncells = -1)
    for (int pass = 0; pass < 3; ++pass) {
        const int lcur = schedule[pass];
        const bool last = pass == 2;
        if (!last && (lcur >= max_lists || max_codes <= 0)) continue;
        const int f1 = std::min(L.l1, lcur), f2 = std::min(L.l2, lcur);
        PSC_TRY(launch_select_probes(d1, nq, idx->imi_k1, f1, marked ? ncells : nullptr, s1, s));
        PSC_TRY(launch_select_probes(d2, nq, idx->imi_k2, f2, marked ? ncells : nullptr, s2, s));
        PSC_TRY(launch_imi_cells(s1, d1, idx->imi_k1, f1, s2, d2, idx->imi_k2, f2, max_lists, lcur, marked, max_codes,
                                 idx->imi_off_dev, nq, cells, ncells, (int *)workspace_dev, s));
        marked = true;
    }
    if (cells_out_dev)
        PSC_HIP_TRY(hipMemcpyAsync(cells_out_dev, cells, (size_t)nq * max_lists * sizeof(int32_t),
                                   hipMemcpyDeviceToDevice, s));
    // 3. the queries' share of the residual tables; 4. one workgroup per query over its cells
    const float *tab1 = nullptr, *tab2 = nullptr;
    if (!L.direct) {
        RowMap map;
        map.sub = im.origin;
        PSC_TRY(launch_lut(idx->cb_dev, idx->dim, idx->m, q_dev, nq, map, true, lut, s));
        PSC_TRY(sync_imi_tables(idx, s));
        tab1 = idx->imi_tab_dev;
        tab2 = tab1 + (size_t)idx->imi_k1 * (idx->m / 2) * kCentroids;
    }
    return launch_imi_scan(idx->m, lut, tab1, tab2, idx->cb_dev, q_dev, im.c1, im.c2, idx->dim, idx->imi_k2, cells,
                           ncells, max_lists, idx->imi_off_dev, idx->imi_codes_dev, idx->imi_ids_dev, ht, k, L.direct,
                           nq, qcodes_out_dev, ids_dev, dists_dev, L.split, (float *)(w + L.off_part_d),
                           (int64_t *)(w + L.off_part_i), (const int *)workspace_dev, s);
}

int psc_workspace_status(void *workspace_dev, psc_stream stream)
{
    PSC_REQUIRE(workspace_dev != nullptr, "null workspace");
    int flag = 0;
    PSC_HIP_TRY(hipMemcpyAsync(&flag, workspace_dev, sizeof(int), hipMemcpyDeviceToHost, (hipStream_t)stream));
    PSC_HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
    if (flag != 0) {
        set_error("a scan gave up on an internal wait; its results are invalid");
        return PSC_EHIP;
    }
    return PSC_OK;
}

}  // extern "C"
