// Host-side training: Lloyd k-means for the product quantizer (Section 3, opening) and the
// index-assignment optimisation by simulated annealing (Sections 3.1 and 3.2).
// Runs once, offline; the search path never comes here.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <limits>
#include <numeric>
#include <thread>

#include "common.h"

namespace psc {
namespace {

// SplitMix64 output function on a counter: draw number `c` of stream `seed`.
inline uint64_t counter_draw(uint64_t seed, uint64_t c)
{
    uint64_t z = seed + 0x9E3779B97F4A7C15ULL * (c + 1);
    z ^= z >> 30;
    z *= 0xBF58476D1CE4E5B9ULL;
    z ^= z >> 27;
    z *= 0x94D049BB133111EBULL;
    z ^= z >> 31;
    return z;
}

template <class F>
void parallel_rows(int64_t n, F &&body)
{
    unsigned hw = std::thread::hardware_concurrency();
    int nt = (int)std::min<int64_t>(std::max(1u, std::min(hw, 32u)), std::max<int64_t>(1, n / 1024));
    if (nt <= 1) {
        body(0, n);
        return;
    }
    std::vector<std::thread> pool;
    int64_t per = (n + nt - 1) / nt;
    for (int t = 0; t < nt; ++t) {
        int64_t lo = t * per, hi = std::min(n, lo + per);
        if (lo >= hi) break;
        pool.emplace_back([&body, lo, hi] { body(lo, hi); });
    }
    for (auto &th : pool) th.join();
}

}  // namespace

// The start of k-means: ncent distinct rows out of n (partial Fisher-Yates on the row numbers,
// draw c of the counter-based generator picks the c-th row).
void kmeans_start_rows(int64_t n, int ncent, uint64_t seed, int64_t *rows)
{
    std::vector<int64_t> perm((size_t)n);
    std::iota(perm.begin(), perm.end(), (int64_t)0);
    for (int c = 0; c < ncent; ++c) {
        int64_t r = c + (int64_t)(counter_draw(seed, (uint64_t)c) % (uint64_t)(n - c));
        std::swap(perm[(size_t)c], perm[(size_t)r]);
        rows[c] = perm[(size_t)c];
    }
}

int host_kmeans(const float *x, int64_t n, int d, int ncent, int iters, uint64_t seed, float *cent)
{
    if (n < ncent) {
        set_error("k-means needs at least %d training vectors, got %lld", ncent, (long long)n);
        return PSC_EINVAL;
    }
    {
        std::vector<int64_t> rows((size_t)ncent);
        kmeans_start_rows(n, ncent, seed, rows.data());
        for (int c = 0; c < ncent; ++c)
            std::memcpy(cent + (size_t)c * d, x + (size_t)rows[(size_t)c] * d, sizeof(float) * d);
    }
    std::vector<int32_t> assign(n);
    std::vector<float> dmin(n);
    std::vector<double> sum((size_t)ncent * d);
    std::vector<int64_t> count(ncent);
    for (int it = 0; it < iters; ++it) {
        parallel_rows(n, [&](int64_t lo, int64_t hi) {
            for (int64_t i = lo; i < hi; ++i) {
                const float *xi = x + (size_t)i * d;
                float best = std::numeric_limits<float>::infinity();
                int bi = 0;
                for (int c = 0; c < ncent; ++c) {
                    const float *cc = cent + (size_t)c * d;
                    float acc = 0.f;
                    for (int t = 0; t < d; ++t) {
                        float df = xi[t] - cc[t];
                        acc += df * df;
                    }
                    if (acc < best) {
                        best = acc;
                        bi = c;
                    }
                }
                assign[i] = bi;
                dmin[i] = best;
            }
        });
        std::fill(sum.begin(), sum.end(), 0.0);
        std::fill(count.begin(), count.end(), (int64_t)0);
        for (int64_t i = 0; i < n; ++i) {
            double *s = sum.data() + (size_t)assign[i] * d;
            const float *xi = x + (size_t)i * d;
            for (int t = 0; t < d; ++t) s[t] += xi[t];
            ++count[assign[i]];
        }
        // empty cells: each takes the member of the (currently) most populated cell that lies
        // farthest from that cell's centroid; the donor's own mean is left as computed
        std::vector<int64_t> pop(count);
        for (int c = 0; c < ncent; ++c) {
            if (pop[c] != 0) continue;
            int big = (int)(std::max_element(pop.begin(), pop.end()) - pop.begin());
            int64_t far = -1;
            float fd = -1.f;
            for (int64_t i = 0; i < n; ++i)
                if (assign[i] == big && dmin[i] > fd) {
                    fd = dmin[i];
                    far = i;
                }
            if (far < 0) continue;
            const float *xf = x + (size_t)far * d;
            for (int t = 0; t < d; ++t) sum[(size_t)c * d + t] = xf[t];
            count[c] = 1;
            --pop[big];
            pop[c] = 1;
            assign[far] = c;
            dmin[far] = 0.f;
        }
        for (int c = 0; c < ncent; ++c)
            if (count[c] > 0)
                for (int t = 0; t < d; ++t)
                    cent[(size_t)c * d + t] = (float)(sum[(size_t)c * d + t] / (double)count[c]);
    }
    return PSC_OK;
}

// ---------------------------------------------------------------------------------------------
// Index assignment.  State kept as the inverse view too would not help: the loss change of a
// transposition touches one row/column pair, O(256).
// ---------------------------------------------------------------------------------------------
namespace {

struct Objective {
    // target = f(d_ij): centroid distances mapped linearly onto the Hamming range so that they
    // share the mean nbit/2 and variance nbit/4 of distances between random nbit-bit strings;
    // weight = alpha^target (Section 3.1).
    std::vector<double> target, weight;
    uint8_t hd[kCentroids][kCentroids];  // Hamming distance between 8-bit indices

    Objective(const float *cent, int dsub, double alpha)
        : target((size_t)kCentroids * kCentroids), weight((size_t)kCentroids * kCentroids)
    {
        const int nbit = 8;
        for (int a = 0; a < kCentroids; ++a)
            for (int b = 0; b < kCentroids; ++b) hd[a][b] = (uint8_t)__builtin_popcount(a ^ b);
        std::vector<double> dist((size_t)kCentroids * kCentroids);
        double s1 = 0.0;
        for (int i = 0; i < kCentroids; ++i)
            for (int j = 0; j < kCentroids; ++j) {
                double acc = 0.0;
                for (int t = 0; t < dsub; ++t) {
                    double df = (double)cent[(size_t)i * dsub + t] - (double)cent[(size_t)j * dsub + t];
                    acc += df * df;
                }
                dist[(size_t)i * kCentroids + j] = std::sqrt(acc);
                if (i != j) s1 += dist[(size_t)i * kCentroids + j];
            }
        const double npairs = (double)kCentroids * (kCentroids - 1);
        const double mu = s1 / npairs;
        double s2 = 0.0;
        for (int i = 0; i < kCentroids; ++i)
            for (int j = 0; j < kCentroids; ++j)
                if (i != j) {
                    double e = dist[(size_t)i * kCentroids + j] - mu;
                    s2 += e * e;
                }
        const double sigma = std::sqrt(s2 / npairs);
        const double slope = std::sqrt((double)nbit) / (2.0 * sigma);
        for (size_t e = 0; e < dist.size(); ++e) {
            target[e] = slope * (dist[e] - mu) + (double)nbit / 2.0;
            weight[e] = std::pow(alpha, target[e]);
        }
    }

    double loss(const uint8_t *pi) const
    {
        double L = 0.0;
        for (int i = 0; i < kCentroids; ++i)
            for (int j = 0; j < kCentroids; ++j) {
                double e = (double)hd[pi[i]][pi[j]] - target[(size_t)i * kCentroids + j];
                L += weight[(size_t)i * kCentroids + j] * e * e;
            }
        return L;
    }

    // Change of the loss when centroids a and b exchange their indices.
    double transposition_delta(const uint8_t *pi, int a, int b) const
    {
        const double *ta = &target[(size_t)a * kCentroids], *tb = &target[(size_t)b * kCentroids];
        const double *wa = &weight[(size_t)a * kCentroids], *wb = &weight[(size_t)b * kCentroids];
        const uint8_t *ha = hd[pi[a]], *hb = hd[pi[b]];
        double acc = 0.0;
        for (int k = 0; k < kCentroids; ++k) {
            if (k == a || k == b) continue;
            double da = (double)ha[pi[k]], db = (double)hb[pi[k]];
            acc += wa[k] * ((db - ta[k]) * (db - ta[k]) - (da - ta[k]) * (da - ta[k]));
            acc += wb[k] * ((da - tb[k]) * (da - tb[k]) - (db - tb[k]) * (db - tb[k]));
        }
        return 2.0 * acc;
    }
};

}  // namespace

namespace {

// The ranking objective of Section 3.1: sum over ordered pairs (i, j), j != i, of
// alpha_rank(i,j) * ell_{r_pi(i,j)}, alpha_r = 1/r, ell_r = 1 + 1/2 + ... + 1/r, where rank(i,j)
// is the place of j among the centroids ordered by distance to i (the nearest other centroid has
// rank 1) and r_pi(i,j) counts the centroids k that are farther from i than j by centroid
// distance yet nearer than j by Hamming distance between indices.
// Sets of centroids are 256-bit masks: far[i][j] = {k : d_ij < d_ik} is fixed; for the current
// assignment nearer[i][h] = {k : h(pi_i, pi_k) < h}, so r_pi(i,j) = |far[i][j] & nearer[i][h(pi_i,pi_j)]|
// -- four and/popcount steps -- and a proposal is scored by recounting every pair.
struct RankingObjective {
    struct Mask {
        uint64_t w[4];
    };
    std::vector<Mask> far;           // [256][256]
    std::vector<int32_t> rank;       // [256][256]
    std::vector<uint16_t> viol;      // [256][256] r_pi of the current assignment
    std::vector<Mask> nearer;        // [256][9]
    double ell[kCentroids + 1];
    uint8_t hd[kCentroids][kCentroids];

    RankingObjective(const float *cent, int dsub)
        : far((size_t)kCentroids * kCentroids), rank((size_t)kCentroids * kCentroids),
          viol((size_t)kCentroids * kCentroids), nearer((size_t)kCentroids * 9)
    {
        for (int a = 0; a < kCentroids; ++a)
            for (int b = 0; b < kCentroids; ++b) hd[a][b] = (uint8_t)__builtin_popcount(a ^ b);
        ell[0] = 0.0;
        for (int r = 1; r <= kCentroids; ++r) {  // each ell_r summed from 1/1 upwards
            double acc = 0.0;
            for (int t = 1; t <= r; ++t) acc += 1.0 / (double)t;
            ell[r] = acc;
        }
        std::vector<double> dist((size_t)kCentroids * kCentroids);
        for (int i = 0; i < kCentroids; ++i)
            for (int j = 0; j < kCentroids; ++j) {
                double acc = 0.0;
                for (int t = 0; t < dsub; ++t) {
                    double df = (double)cent[(size_t)i * dsub + t] - (double)cent[(size_t)j * dsub + t];
                    acc += df * df;
                }
                dist[(size_t)i * kCentroids + j] = std::sqrt(acc);
            }
        for (int i = 0; i < kCentroids; ++i)
            for (int j = 0; j < kCentroids; ++j) {
                Mask f = {{0, 0, 0, 0}};
                int nearer_than_j = 0;
                const double dij = dist[(size_t)i * kCentroids + j];
                for (int k = 0; k < kCentroids; ++k) {
                    const double dik = dist[(size_t)i * kCentroids + k];
                    if (dij < dik) f.w[k >> 6] |= 1ull << (k & 63);
                    nearer_than_j += dik < dij;
                }
                far[(size_t)i * kCentroids + j] = f;
                rank[(size_t)i * kCentroids + j] = nearer_than_j;
            }
    }

    void build_nearer(const uint8_t *pi, std::vector<Mask> &out) const
    {
        for (int i = 0; i < kCentroids; ++i) {
            Mask eq[9];
            std::memset(eq, 0, sizeof eq);
            for (int k = 0; k < kCentroids; ++k) eq[hd[pi[i]][pi[k]]].w[k >> 6] |= 1ull << (k & 63);
            Mask run = {{0, 0, 0, 0}};
            for (int h = 0; h < 9; ++h) {  // nearer[h] = union of eq[0 .. h-1]
                out[(size_t)i * 9 + h] = run;
                for (int w = 0; w < 4; ++w) run.w[w] |= eq[h].w[w];
            }
        }
    }

    static int count(const Mask &a, const Mask &b)
    {
        return __builtin_popcountll(a.w[0] & b.w[0]) + __builtin_popcountll(a.w[1] & b.w[1]) +
               __builtin_popcountll(a.w[2] & b.w[2]) + __builtin_popcountll(a.w[3] & b.w[3]);
    }

    void count_all(const uint8_t *pi, const std::vector<Mask> &nr, std::vector<uint16_t> &out) const
    {
        for (int i = 0; i < kCentroids; ++i)
            for (int j = 0; j < kCentroids; ++j)
                out[(size_t)i * kCentroids + j] =
                    (uint16_t)count(far[(size_t)i * kCentroids + j], nr[(size_t)i * 9 + hd[pi[i]][pi[j]]]);
    }

    void set_assignment(const uint8_t *pi)
    {
        build_nearer(pi, nearer);
        count_all(pi, nearer, viol);
    }

    double loss() const
    {
        double L = 0.0;
        for (int i = 0; i < kCentroids; ++i)
            for (int j = 0; j < kCentroids; ++j) {
                const size_t e = (size_t)i * kCentroids + j;
                if (j == i || rank[e] == 0) continue;
                L += ell[viol[e]] / (double)rank[e];
            }
        return L;
    }
};

}  // namespace

void host_anneal_ranking(const float *cent, int dsub, int64_t n_iter, double t0, double t_decay, uint64_t seed,
                         uint8_t *pi, double *loss_before, double *loss_after)
{
    RankingObjective obj(cent, dsub);
    for (int i = 0; i < kCentroids; ++i) pi[i] = (uint8_t)i;
    obj.set_assignment(pi);
    if (loss_before) *loss_before = obj.loss();
    std::vector<RankingObjective::Mask> nr_try(obj.nearer.size());
    std::vector<uint16_t> viol_try(obj.viol.size());
    double temperature = t0;
    for (int64_t it = 0; it < n_iter; ++it) {
        const uint64_t c = 3 * (uint64_t)it;
        const int a = (int)(counter_draw(seed, c) % kCentroids);
        const int b = (int)((a + 1 + counter_draw(seed, c + 1) % (kCentroids - 1)) % kCentroids);
        const double u = (double)(counter_draw(seed, c + 2) >> 11) * 0x1.0p-53;
        std::swap(pi[a], pi[b]);
        obj.build_nearer(pi, nr_try);
        obj.count_all(pi, nr_try, viol_try);
        double delta = 0.0;  // pairs whose count is unchanged contribute exactly nothing
        for (int i = 0; i < kCentroids; ++i)
            for (int j = 0; j < kCentroids; ++j) {
                const size_t e = (size_t)i * kCentroids + j;
                if (j == i || obj.rank[e] == 0 || viol_try[e] == obj.viol[e]) continue;
                delta += (obj.ell[viol_try[e]] - obj.ell[obj.viol[e]]) / (double)obj.rank[e];
            }
        if (delta < 0.0 || u < temperature) {
            obj.nearer.swap(nr_try);
            obj.viol.swap(viol_try);
        } else {
            std::swap(pi[a], pi[b]);
        }
        temperature *= t_decay;
    }
    if (loss_after) *loss_after = obj.loss();
}

void host_anneal(const float *cent, int dsub, int64_t n_iter, double t0, double t_decay,
                 double alpha, uint64_t seed, uint8_t *pi, double *loss_before, double *loss_after)
{
    Objective obj(cent, dsub, alpha);
    for (int i = 0; i < kCentroids; ++i) pi[i] = (uint8_t)i;
    if (loss_before) *loss_before = obj.loss(pi);
    double temperature = t0;
    for (int64_t it = 0; it < n_iter; ++it) {
        const uint64_t c = 3 * (uint64_t)it;
        const int a = (int)(counter_draw(seed, c) % kCentroids);
        const int b = (int)((a + 1 + counter_draw(seed, c + 1) % (kCentroids - 1)) % kCentroids);
        const double u = (double)(counter_draw(seed, c + 2) >> 11) * 0x1.0p-53;
        const double delta = obj.transposition_delta(pi, a, b);
        if (delta < 0.0 || u < temperature) std::swap(pi[a], pi[b]);
        temperature *= t_decay;
    }
    if (loss_after) *loss_after = obj.loss(pi);
}

}  // namespace psc
