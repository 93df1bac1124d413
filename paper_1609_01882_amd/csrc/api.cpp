// C ABI of libpsc: argument checking and dispatch.  See include/psc.h for the contract.
#include <cstring>
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
    return PSC_OK;
}

static int sync_codebook_to_device(const psc_index *idx)
{
    if (idx->dev_current) return PSC_OK;
    const size_t bytes = idx->cb_host.size() * sizeof(float);
    if (!idx->cb_dev) PSC_HIP_TRY(hipMalloc((void **)&idx->cb_dev, bytes));
    PSC_HIP_TRY(hipMemcpy(idx->cb_dev, idx->cb_host.data(), bytes, hipMemcpyHostToDevice));
    idx->dev_current = true;
    return PSC_OK;
}

}  // namespace psc

using namespace psc;

extern "C" {

int psc_version(void) { return 100; }

const char *psc_last_error(void) { return g_error.c_str(); }

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

int psc_optimize_index_assignment(psc_index *idx, int64_t n_iter, double t0, double t_decay,
                                  double alpha, uint64_t seed, uint8_t *perm_out_host,
                                  double *loss_out_host)
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
    rc = launch_lut(idx->cb_dev, idx->dim, idx->m, q_dev, nq, RowMap{}, lut_dev, (hipStream_t)stream);
    if (rc != PSC_OK) return rc;
    if (qcodes_dev)
        rc = launch_encode(idx->cb_dev, idx->dim, idx->m, q_dev, nq, RowMap{}, qcodes_dev, (hipStream_t)stream);
    return rc;
}

int psc_hamming_filter(int m, const uint8_t *qcodes_dev, int64_t nq, const uint8_t *codes_dev,
                       int64_t n, int ht, int64_t *nsurv_dev, uint8_t *hdist_dev, psc_stream stream)
{
    return launch_hamming_filter(m, qcodes_dev, nq, codes_dev, n, ht, nsurv_dev, hdist_dev, (hipStream_t)stream);
}

size_t psc_scan_workspace_bytes(int m, int64_t nq, int64_t n, int k)
{
    ScanPlan p;
    if (plan_scan(m, nq, n, k, &p) != PSC_OK) return 0;
    return p.total_bytes;
}

int psc_scan(int m, const float *lut_dev, const uint8_t *qcodes_dev, int64_t nq,
             const uint8_t *codes_dev, int64_t n, int ht, int k, int64_t *ids_dev,
             float *dists_dev, void *workspace_dev, size_t workspace_bytes, psc_stream stream)
{
    return launch_scan(m, lut_dev, qcodes_dev, nq, codes_dev, n, ht, k, -1, true, ids_dev, dists_dev,
                       workspace_dev, workspace_bytes, (hipStream_t)stream);
}

static size_t round256(size_t v) { return (v + 255) / 256 * 256; }

size_t psc_search_workspace_bytes(const psc_index *idx, int64_t nq, int64_t n, int k)
{
    if (!idx) return 0;
    ScanPlan p;
    if (plan_scan(idx->m, nq, n, k, &p) != PSC_OK) return 0;
    return round256(p.total_bytes) + round256((size_t)nq * idx->m * kCentroids * sizeof(float)) +
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
    ScanPlan p;
    rc = plan_scan(idx->m, nq, n, k, &p);
    if (rc != PSC_OK) return rc;
    char *w = (char *)workspace_dev + round256(p.total_bytes);
    float *lut = (float *)w;
    w += round256((size_t)nq * idx->m * kCentroids * sizeof(float));
    uint8_t *qcodes = (uint8_t *)w;
    rc = psc_build_lut(idx, q_dev, nq, lut, qcodes, stream);
    if (rc != PSC_OK) return rc;
    return launch_scan(idx->m, lut, qcodes, nq, codes_dev, n, ht, k, -1, true, ids_dev, dists_dev,
                       workspace_dev, round256(p.total_bytes), (hipStream_t)stream);
}

// ---------------------------------------------------------------------------------------------
// k-NN graph (Section 5): every database vector in turn is the query.  Queries are processed in
// chunks so that one chunk's tables fit the workspace; each chunk is a flat scan whose query
// codes are the stored codes of the chunk's rows and which never returns a row to itself.
// ---------------------------------------------------------------------------------------------
static const int64_t kGraphChunk = 32768;

// Scan workspace that serves both the full chunks and the shorter last chunk (whose plan may
// cut the database into more slices).
static size_t graph_scan_workspace(const psc_index *idx, int64_t n, int k)
{
    const int64_t qc = n < kGraphChunk ? n : kGraphChunk;
    const int64_t tail = n % kGraphChunk;
    ScanPlan p, pt;
    if (plan_scan(idx->m, qc, n, k, &p) != PSC_OK) return 0;
    size_t bytes = p.total_bytes;
    if (n > kGraphChunk && tail != 0) {
        if (plan_scan(idx->m, tail, n, k, &pt) != PSC_OK) return 0;
        if (pt.total_bytes > bytes) bytes = pt.total_bytes;
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
    const int64_t qc_max = n < kGraphChunk ? n : kGraphChunk;
    const size_t scan_ws_bytes = graph_scan_workspace(idx, n, k);
    char *scan_ws = (char *)workspace_dev;
    float *lut = (float *)((char *)workspace_dev + scan_ws_bytes);
    for (int64_t c0 = 0; c0 < n; c0 += kGraphChunk) {
        const int64_t qc = (n - c0) < kGraphChunk ? (n - c0) : kGraphChunk;
        rc = launch_lut(idx->cb_dev, idx->dim, idx->m, x_dev + (size_t)c0 * idx->dim, qc, RowMap{}, lut,
                        (hipStream_t)stream);
        if (rc != PSC_OK) return rc;
        rc = launch_scan(idx->m, lut, codes_dev + (size_t)c0 * idx->m, qc, codes_dev, n, ht, k, c0, c0 == 0,
                         ids_dev + (size_t)c0 * k, dists_dev + (size_t)c0 * k, scan_ws, scan_ws_bytes,
                         (hipStream_t)stream);
        if (rc != PSC_OK) return rc;
    }
    return PSC_OK;
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
