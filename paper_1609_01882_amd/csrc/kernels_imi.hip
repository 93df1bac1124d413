// Inverted multi-index (Section 2 "Non-exhaustive search"; Section 4.3; caption of Table 2).
//
// The coarse level is a product quantizer: the first half of a vector is quantized with K1
// centroids, the second half with K2, which gives K1*K2 cells; cell (a, b) has number a*K2 + b and
// centroid (c1[a], c2[b]).  A query visits cells in non-decreasing order of its squared distance
// to the cell centroid, d1[a] + d2[b] (lower cell number first on equal sums), until max_lists
// cells are taken or the cells taken hold max_codes codes or more.  Inside a cell the search is
// the polysemous one on residuals: bit string and ADC tables from q - (c1[a], c2[b]).
//
// Work here is shaped differently from the plain inverted file: with K1*K2 in the millions a cell
// holds a handful of codes and hardly two queries of a batch meet in one, so nothing is grouped by
// cell.  One workgroup serves one query from the first cell to the last:
//   * imi_cells_kernel: the L nearest centroids of each half arrive sorted (the inverted file's
//     probe selection, run once per half); the cell at places (i, j) of the two sorted lists has at
//     least (i+1)(j+1)-1 cells in front of it, so only the pairs with (i+1)(j+1) <= L can be among
//     the first L cells (about L ln L of them): their sums are sorted in LDS, which gives the
//     multi-sequence order without a priority queue; the caps are applied to the sorted prefix;
//   * imi_scan_kernel: per cell the residual table is put together in LDS from the query's share
//     ||c||^2 - 2 (q-o).c, the two half-centroids' shares 2 (c1[a]-o1).c and 2 (c2[b]-o2).c -- which
//     depend on a alone for the first m/2 sub-quantizers and on b alone for the others, so K1 + K2
//     half tables replace K1*K2 cell tables -- and ||(q - cell centroid)_j||^2; its row minima give
//     the bit string; the cell's codes are tested 256 at a time, survivors scored from the LDS
//     table and appended to a pool of sortable 64-bit keys (distance, id) that is sorted and cut
//     back to the best k whenever it runs full.
#include "common.h"

namespace psc {
namespace {

#define PSC_LDS __attribute__((address_space(3)))

// float -> unsigned key with the same order (also for negative values, which rounding can produce
// for a distance that should be zero), and back
__device__ __forceinline__ uint32_t fkey(float v)
{
    const uint32_t u = __float_as_uint(v);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float fkey_value(uint32_t k)
{
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

// Smallest value of v over the wave, in every lane: four row-local steps on the data-parallel
// path, then the four row results through scalar registers.
__device__ __forceinline__ uint32_t wave_min_key(uint32_t v)
{
    auto step = [](uint32_t x, uint32_t y) { return y < x ? y : x; };
    v = step(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0xB1, 0xf, 0xf, false));   // lane ^ 1
    v = step(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x4E, 0xf, 0xf, false));   // lane ^ 2
    v = step(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x141, 0xf, 0xf, false));  // mirror in 8
    v = step(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x140, 0xf, 0xf, false));  // mirror in 16
    const uint32_t r0 = (uint32_t)__builtin_amdgcn_readlane((int)v, 0);
    const uint32_t r1 = (uint32_t)__builtin_amdgcn_readlane((int)v, 16);
    const uint32_t r2 = (uint32_t)__builtin_amdgcn_readlane((int)v, 32);
    const uint32_t r3 = (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
    return step(step(r0, r1), step(r2, r3));
}

// Sum of v over the wave, the same in every lane (the same steps as wave_min_key).
__device__ __forceinline__ float wave_sum_f32(float v)
{
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xf, 0xf, false));   // lane ^ 1
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xf, 0xf, false));   // lane ^ 2
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xf, 0xf, false));  // mirror in 8
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xf, 0xf, false));  // mirror in 16
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
    const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
    const float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
    return (r0 + r1) + (r2 + r3);
}

// Ascending bitonic sort of n (a power of two) 64-bit keys in LDS by the whole workgroup.
// With one pair per thread (n <= 2 * blockDim) wave w only touches keys 128 w .. 128 w + 127 in the
// steps whose partners lie 64 places or less apart, and LDS serves a wave's accesses in the order
// they were issued: such steps need no workgroup barrier between them, only the ones around a
// step that reaches across waves do (3 of the 45 steps of a 512-key sort).
__device__ __forceinline__ void bitonic_sort(unsigned long long *keys, int n)
{
    const bool one_pair = n <= 2 * (int)blockDim.x;  // (uniform)
    bool across = true;                              // the step before this one reached across waves
    for (int size = 2; size <= n; size <<= 1)
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            const bool wide = !one_pair || stride > 64;
            if (wide || across) {
                __syncthreads();
            } else {
                __atomic_signal_fence(__ATOMIC_SEQ_CST);
                __builtin_amdgcn_wave_barrier();
            }
            across = wide;
            for (int t = (int)threadIdx.x; t < n / 2; t += (int)blockDim.x) {
                const int lo = 2 * t - (t & (stride - 1));  // t with a zero inserted at bit `stride`
                const int hi = lo + stride;
                const bool up = (lo & size) == 0;
                const unsigned long long a = keys[lo], b = keys[hi];
                if ((a > b) == up) {
                    keys[lo] = b;
                    keys[hi] = a;
                }
            }
        }
    __syncthreads();
}

__global__ void split_halves_kernel(const float *__restrict__ x, int64_t n, int dim, float *__restrict__ h1,
                                    float *__restrict__ h2)
{
    const int half = dim / 2;
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n * dim) return;
    const int64_t r = e / dim;
    const int t = (int)(e - r * dim);
    if (t < half)
        h1[r * half + t] = x[e];
    else
        h2[r * half + t - half] = x[e];
}

__global__ void combine_cells_kernel(const int32_t *__restrict__ a, const int32_t *__restrict__ b, int64_t n, int k2,
                                     int32_t *__restrict__ cell)
{
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e < n) cell[e] = a[e] * k2 + b[e];
}

// One workgroup per query.  sel1 [nq][l1] / sel2 [nq][l2]: the nearest half-centroids in ascending
// (distance, number); dist1 [nq][k1] / dist2 [nq][k2]: all half distances.  Dynamic LDS: npad keys
// (npad = the candidate count rounded up to a power of two), then l1 + 1 ints, then lcur int64.
// The order is found for the first lcur <= lmax cells (candidates: (i+1)(j+1) <= lcur).  A pass
// that is not the last one (lcur < lmax) settles the queries whose cap on codes is reached within
// those cells -- with cells of hundreds of codes that is nearly all of them, at a fraction of the
// sorting work -- and marks the others with ncells = -1; the last pass (lcur = lmax) then takes
// only the marked ones (only_marked), or every query if it is the only pass.
__global__ void __launch_bounds__(256)
imi_cells_kernel(const int32_t *__restrict__ sel1, const float *__restrict__ dist1, int k1, int l1,
                 const int32_t *__restrict__ sel2, const float *__restrict__ dist2, int k2, int l2, int lmax, int lcur,
                 int only_marked, int64_t max_codes, const int64_t *__restrict__ offsets, int npad,
                 int32_t *__restrict__ cells, int32_t *__restrict__ ncells, int *__restrict__ status)
{
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned long long *keys = (unsigned long long *)smem;
    int *pre = (int *)(keys + npad);                     // pre[i] = candidates of rows 0 .. i-1
    long long *held = (long long *)(pre + ((l1 + 2) & ~1));  // codes of the sorted cells
    const int64_t q = blockIdx.x;
    const int tid = (int)threadIdx.x;
    if (q == 0 && tid == 0 && status) *status = 0;  // (nothing in this search waits on anything: always clean)
    if (only_marked && ncells[q] >= 0) return;      // (settled by the pass before; uniform over the workgroup)
    if (tid == 0) {
        int run = 0;
        for (int i = 0; i < l1; ++i) {
            pre[i] = run;
            const int jm = lcur / (i + 1);
            run += jm < l2 ? jm : l2;
        }
        pre[l1] = run;
    }
    __syncthreads();
    const int nc = pre[l1];
    for (int e = tid; e < npad; e += 256) {
        unsigned long long key = ~0ull;
        if (e < nc) {
            int lo = 0, hi = l1 - 1;  // the row i with pre[i] <= e < pre[i+1]
            while (lo < hi) {
                const int mid = (lo + hi + 1) >> 1;
                if (pre[mid] <= e) lo = mid; else hi = mid - 1;
            }
            const int i = lo, j = e - pre[lo];
            const int a = sel1[q * l1 + i], b = sel2[q * l2 + j];
            const float sum = dist1[q * k1 + a] + dist2[q * k2 + b];
            key = ((unsigned long long)fkey(sum) << 32) | (unsigned)(a * k2 + b);
        }
        keys[e] = key;
    }
    bitonic_sort(keys, npad);
    const int lc = nc < lcur ? nc : lcur;
    for (int t = tid; t < lc; t += 256) {
        const int64_t cell = (int64_t)(uint32_t)keys[t];
        held[t] = offsets[cell + 1] - offsets[cell];
    }
    __syncthreads();
    __shared__ int ntake_s;
    if (tid == 0) {  // the caps, on the sorted prefix (at most 1024 steps over LDS)
        long long total = 0;
        int t = 0;
        while (t < lc && !(max_codes > 0 && total >= max_codes)) total += held[t++];
        // not the last pass, and the cap on codes is not reached within these cells: the cells after
        // them are needed, leave the query to the next pass
        if (lcur < lmax && !(max_codes > 0 && total >= max_codes)) t = -1;
        ntake_s = t;
        ncells[q] = t;
    }
    __syncthreads();
    const int ntake = ntake_s;
    if (ntake < 0) return;
    for (int t = tid; t < lmax; t += 256) cells[q * lmax + t] = t < ntake ? (int32_t)(uint32_t)keys[t] : -1;
}

struct ImiScanArgs {
    const float *lut;        // [nq][M][256] the queries' share ||c||^2 - 2 (q-o).c (unused when direct)
    const float *tab1;       // [k1][M/2][256] 2 (c1[a]-o1)_j . c
    const float *tab2;       // [k2][M/2][256]
    const float *cb;         // [M][256][dsub] (direct tables only)
    const float *queries;    // [nq][dim]
    const float *c1, *c2;    // [k1][dim/2], [k2][dim/2]
    const int32_t *cells;    // [nq][lmax], -1 padded
    const int32_t *ncells;   // [nq]
    const int64_t *offsets;  // [k1*k2+1]
    const uint8_t *codes;    // [n][M]
    const int32_t *ext_ids;  // [n]
    uint8_t *qcodes_out;     // [nq][lmax][M] or null
    int64_t *ids;            // [nq][k]            (split == 1)
    float *dists;            // [nq][k]
    int64_t *part_i;         // [nq][split][k]     (split > 1: one list per workgroup, merged afterwards)
    float *part_d;           // [nq][split][k]
    int dim, k2, lmax, ht, k, cap, direct;
    int split;               // workgroups per query: workgroup s of a query takes its cells s, s + split, ...
};

// Dynamic LDS: [M][256] query share, [M][256] cell table, dim floats (residual; dim is even), cap keys.
//
// A cell is short work behind several trips to memory (its bounds, its two half-centroids, its
// two half tables, its codes), so the trips are taken off the path of the cell they belong to: the
// bounds of the workgroup's next kWindow cells are staged in LDS at once, and while one cell is
// worked on every thread already holds, in registers, what it will need of the next one (its
// element of the residual, its entry of each table row, its code of the first step).
template <int M>
__global__ void __launch_bounds__(256)
imi_scan_kernel(ImiScanArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    float *tq = (float *)smem;
    float *cellt = tq + M * 256;
    float *res = cellt + M * 256;
    unsigned long long *pool = (unsigned long long *)(res + a.dim);
    constexpr int kWindow = 32;
    __shared__ int count_s;
    __shared__ uint32_t qcw[M / 4];
    __shared__ float thr_s;
    __shared__ int win_cell[kWindow];
    __shared__ long long win_begin[kWindow], win_end[kWindow];
    const int64_t q = blockIdx.x / a.split;
    const int sub = (int)(blockIdx.x - q * a.split);
    const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = a.dim / 2, dsub = a.dim / M;
    constexpr int WPC = M / 4;
    constexpr int RPW = M / 4;  // table rows per wave: wave w builds rows w * RPW .. and finds their minima alone

    if (!a.direct)
        for (int e = tid; e < M * 64; e += 256)
            ((float4 *)tq)[e] = ((const float4 *)(a.lut + q * (M * 256)))[e];
    for (int e = tid; e < a.cap; e += 256) pool[e] = ~0ull;
    if (tid == 0) {
        count_s = 0;
        thr_s = __builtin_inff();
    }
    const int ncell = a.ncells[q];
    const int mine = ncell > sub ? (ncell - sub + a.split - 1) / a.split : 0;  // cells sub, sub + split, ...
    const float qv = tid < a.dim ? a.queries[q * a.dim + tid] : 0.f;           // the thread's element of the query

    // what a thread holds of a cell before the cell's turn
    struct Inputs {
        float g;            // its element of the cell centroid (tid < dim)
        float th[M];        // its entries of the half tables' rows (not direct): rows of its wave, four each
        uint32_t cw[WPC];   // its code of the cell's first 256
        int32_t id;         // and that code's id
    };
    auto fetch = [&](int w, Inputs &in) {  // w: place in the window
        const int cell = win_cell[w];
        in.g = 0.f;
#pragma unroll
        for (int jj = 0; jj < M; ++jj) in.th[jj] = 0.f;
#pragma unroll
        for (int ww = 0; ww < WPC; ++ww) in.cw[ww] = 0u;
        in.id = 0;
        if (cell < 0) return;
        const int ca = cell / a.k2, cb_ = cell - ca * a.k2;
        if (tid < a.dim) in.g = tid < half ? a.c1[(int64_t)ca * half + tid] : a.c2[(int64_t)cb_ * half + tid - half];
        if (!a.direct) {
#pragma unroll
            for (int r = 0; r < RPW; ++r) {
                const int jj = wave * RPW + r;  // (a wave's rows lie in one half: RPW divides M / 2)
                const float *row = jj < M / 2 ? a.tab1 + ((int64_t)ca * (M / 2) + jj) * 256
                                              : a.tab2 + ((int64_t)cb_ * (M / 2) + jj - M / 2) * 256;
#pragma unroll
                for (int c = 0; c < 4; ++c) in.th[r * 4 + c] = row[c * 64 + lane];
            }
        }
        const long long i = win_begin[w] + tid;
        if (i < win_end[w]) {
            const uint32_t *src = (const uint32_t *)(a.codes + i * M);
#pragma unroll
            for (int ww = 0; ww < WPC; ++ww) in.cw[ww] = src[ww];
            in.id = a.ext_ids[i];
        }
    };

    for (int base = 0; base < mine; base += kWindow) {
        __syncthreads();  // (the window of the round before is no longer read; first round: the set-up above)
        if (tid < kWindow) {
            int cell = -1;
            long long b = 0, e = 0;
            if (base + tid < mine) {
                cell = a.cells[q * a.lmax + sub + (int64_t)(base + tid) * a.split];
                b = a.offsets[cell];
                e = a.offsets[cell + 1];
            }
            win_cell[tid] = cell;
            win_begin[tid] = b;
            win_end[tid] = e;
        }
        __syncthreads();
        const int nwin = mine - base < kWindow ? mine - base : kWindow;
        Inputs cur, nxt;
        fetch(0, cur);
        for (int w = 0; w < nwin; ++w) {
            const int p = sub + (base + w) * a.split;  // the cell's place in the query's order
            const long long begin = win_begin[w], end = win_end[w];
            if (w + 1 < nwin) fetch(w + 1, nxt);
            if (!(begin == end && !a.qcodes_out)) {  // (uniform over the workgroup)
                // ---- residual to the cell centroid (one element per thread, held since the cell before;
                //      vectors of more than 256 dimensions take theirs from memory here)
                if (a.dim <= 256) {
                    if (tid < a.dim) res[tid] = qv - cur.g;
                } else {
                    const int cell = win_cell[w];
                    const int ca = cell / a.k2, cb_ = cell - ca * a.k2;
                    for (int t = tid; t < a.dim; t += 256)
                        res[t] = a.queries[q * a.dim + t] -
                                 (t < half ? a.c1[(int64_t)ca * half + t] : a.c2[(int64_t)cb_ * half + t - half]);
                }
                __syncthreads();
                // ---- the cell's table: wave w builds rows w * RPW .., four entries of a row per lane;
                //      the row's minimum (lowest index on ties) is the cell's bit string for that row
#pragma unroll
                for (int r = 0; r < RPW; ++r) {
                    const int jj = wave * RPW + r;
                    // || (q - cell centroid)_jj ||^2: a coordinate (or a few) per lane, summed over the wave
                    float part = 0.f;
                    for (int t = lane; t < dsub; t += 64) part = fmaf(res[jj * dsub + t], res[jj * dsub + t], part);
                    const float sq = wave_sum_f32(part);
                    uint32_t best = 0xffffffffu;
                    int besti = 0;
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const int e = c * 64 + lane;
                        float v;
                        if (a.direct) {
                            const float *cr = a.cb + ((int64_t)jj * 256 + e) * dsub;
                            v = 0.f;
                            for (int t = 0; t < dsub; ++t) {
                                const float df = res[jj * dsub + t] - cr[t];
                                v = fmaf(df, df, v);
                            }
                        } else {
                            v = (tq[jj * 256 + e] + cur.th[r * 4 + c]) + sq;
                        }
                        cellt[jj * 256 + e] = v;
                        const uint32_t key = fkey(v);
                        if (key < best) {  // (ascending e: the lowest index stays on ties)
                            best = key;
                            besti = e;
                        }
                    }
                    // the smallest key of the wave, then the lowest index among the lanes that hold it
                    const uint32_t wmin = wave_min_key(best);
                    const uint32_t imin = wave_min_key(best == wmin ? (uint32_t)besti : 0xffffffffu);
                    if (lane == 0) ((volatile uint8_t *)qcw)[jj] = (uint8_t)imin;
                }
                __syncthreads();
                if (a.qcodes_out && tid < M) a.qcodes_out[(q * a.lmax + p) * M + tid] = ((volatile uint8_t *)qcw)[tid];
                uint32_t qw[WPC];
#pragma unroll
                for (int ww = 0; ww < WPC; ++ww) qw[ww] = qcw[ww];
                // ---- the cell's codes, 256 at a time (the first 256 are in registers already; every
                //      step asks for the next one's before it works on its own)
                uint32_t cw[WPC];
#pragma unroll
                for (int ww = 0; ww < WPC; ++ww) cw[ww] = cur.cw[ww];
                int32_t id = cur.id;  // (asked for with the code: a survivor's id is not one more trip to memory)
                for (long long i0 = begin; i0 < end; i0 += 256) {
                    const long long i = i0 + tid;
                    uint32_t nw[WPC];
                    int32_t nid = 0;
#pragma unroll
                    for (int ww = 0; ww < WPC; ++ww) nw[ww] = 0u;
                    if (i + 256 < end) {
                        const uint32_t *src = (const uint32_t *)(a.codes + (i + 256) * M);
#pragma unroll
                        for (int ww = 0; ww < WPC; ++ww) nw[ww] = src[ww];
                        nid = a.ext_ids[i + 256];
                    }
                    if (i < end) {
                        int h = 0;
#pragma unroll
                        for (int ww = 0; ww < WPC; ++ww) h += __builtin_popcount(cw[ww] ^ qw[ww]);
                        if (h <= a.ht) {
                            float d = 0.f;
#pragma unroll
                            for (int jj = 0; jj < M; ++jj) d += cellt[jj * 256 + ((cw[jj >> 2] >> (8 * (jj & 3))) & 0xffu)];
                            if (!(d > thr_s)) {
                                const int at = atomicAdd(&count_s, 1);
                                pool[at] = ((unsigned long long)fkey(d) << 32) | (uint32_t)id;
                            }
                        }
                    }
#pragma unroll
                    for (int ww = 0; ww < WPC; ++ww) cw[ww] = nw[ww];
                    id = nid;
                    __syncthreads();
                    if (count_s > a.cap - 256) {  // (uniform) no room for another step: keep the best k
                        bitonic_sort(pool, a.cap);
                        const int kept = count_s < a.k ? count_s : a.k;
                        for (int e = kept + tid; e < a.cap; e += 256) pool[e] = ~0ull;
                        __syncthreads();
                        if (tid == 0) {
                            count_s = kept;
                            if (kept == a.k) thr_s = fkey_value((uint32_t)(pool[a.k - 1] >> 32));
                        }
                        __syncthreads();
                    }
                }
                // (no barrier here: the next cell writes the residual first, and nothing of this cell is
                //  read after the barrier that ended its last step -- or, without codes, the one above)
            }
            cur = nxt;
        }
    }
    __syncthreads();
    bitonic_sort(pool, a.cap);
    const int found = count_s < a.k ? count_s : a.k;
    int64_t *ids = a.split > 1 ? a.part_i + (q * a.split + sub) * a.k : a.ids + q * a.k;
    float *dists = a.split > 1 ? a.part_d + (q * a.split + sub) * a.k : a.dists + q * a.k;
    for (int r = tid; r < a.k; r += 256) {
        const unsigned long long key = pool[r];
        ids[r] = r < found ? (int64_t)(int32_t)(uint32_t)key : -1;
        dists[r] = r < found ? fkey_value((uint32_t)(key >> 32)) : __builtin_inff();
    }
}

}  // namespace

int launch_split_halves(const float *x_dev, int64_t n, int dim, float *h1_dev, float *h2_dev, hipStream_t s)
{
    const int64_t total = n * dim;
    if (total == 0) return PSC_OK;
    PSC_REQUIRE((total + 255) / 256 <= 0x7fffffffLL, "too many rows");
    hipLaunchKernelGGL(split_halves_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, x_dev, n, dim, h1_dev,
                       h2_dev);
    PSC_HIP_TRY(hipGetLastError());
    return PSC_OK;
}

int launch_combine_cells(const int32_t *a_dev, const int32_t *b_dev, int64_t n, int k2, int32_t *cell_dev, hipStream_t s)
{
    if (n == 0) return PSC_OK;
    hipLaunchKernelGGL(combine_cells_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, a_dev, b_dev, n, k2,
                       cell_dev);
    PSC_HIP_TRY(hipGetLastError());
    return PSC_OK;
}

// Candidate pairs (i, j) with (i+1)(j+1) <= lmax inside an l1 x l2 grid.
static int64_t imi_candidates(int l1, int l2, int lmax)
{
    int64_t nc = 0;
    for (int i = 0; i < l1; ++i) nc += std::min<int64_t>(lmax / (i + 1), l2);
    return nc;
}

int launch_imi_cells(const int32_t *sel1_dev, const float *dist1_dev, int k1, int l1, const int32_t *sel2_dev,
                     const float *dist2_dev, int k2, int l2, int lmax, int lcur, bool only_marked, int64_t max_codes,
                     const int64_t *offsets_dev, int64_t nq, int32_t *cells_dev, int32_t *ncells_dev, int *status_dev,
                     hipStream_t s)
{
    if (nq == 0) return PSC_OK;
    PSC_REQUIRE(lmax >= 1 && lmax <= 1024 && lcur >= 1 && lcur <= lmax && l1 >= 1 && l2 >= 1 && nq <= 0x7fffffffLL,
                "bad multi-index shape");
    static bool configured = false;
    if (!configured) {
        // (up to 8192 keys + 1026 ints + 1024 counts; the kernel also has a few static words)
        PSC_HIP_TRY(hipFuncSetAttribute((const void *)imi_cells_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                        96 * 1024));
        configured = true;
    }
    const int64_t nc = imi_candidates(l1, l2, lcur);
    int npad = 2;
    while (npad < nc) npad <<= 1;
    const size_t lds = (size_t)npad * 8 + (size_t)((l1 + 2) & ~1) * 4 + (size_t)lcur * 8;
    PSC_REQUIRE(lds <= 96 * 1024, "too many candidate cells");
    hipLaunchKernelGGL(imi_cells_kernel, dim3((unsigned)nq), dim3(256), lds, s, sel1_dev, dist1_dev, k1, l1, sel2_dev,
                       dist2_dev, k2, l2, lmax, lcur, only_marked ? 1 : 0, max_codes, offsets_dev, npad, cells_dev,
                       ncells_dev, status_dev);
    PSC_HIP_TRY(hipGetLastError());
    return PSC_OK;
}

int launch_imi_scan(int m, const float *lut_dev, const float *tab1_dev, const float *tab2_dev, const float *cb_dev,
                    const float *queries_dev, const float *c1_dev, const float *c2_dev, int dim, int k2,
                    const int32_t *cells_dev, const int32_t *ncells_dev, int lmax, const int64_t *offsets_dev,
                    const uint8_t *codes_dev, const int32_t *ext_ids_dev, int ht, int k, bool direct, int64_t nq,
                    uint8_t *qcodes_out_dev, int64_t *ids_dev, float *dists_dev, int split, float *part_d_dev,
                    int64_t *part_i_dev, const int *status_dev, hipStream_t s)
{
    if (nq == 0) return PSC_OK;
    PSC_REQUIRE(split >= 1 && nq * split <= 0x7fffffffLL, "too many queries");
    PSC_REQUIRE(split == 1 || (part_d_dev && part_i_dev && status_dev), "no room for the partial lists");
    PSC_REQUIRE(((uintptr_t)codes_dev & 15) == 0 && ((uintptr_t)lut_dev & 15) == 0, "codes and tables must be 16-byte aligned");
    ImiScanArgs a;
    a.lut = lut_dev;
    a.tab1 = tab1_dev;
    a.tab2 = tab2_dev;
    a.cb = cb_dev;
    a.queries = queries_dev;
    a.c1 = c1_dev;
    a.c2 = c2_dev;
    a.cells = cells_dev;
    a.ncells = ncells_dev;
    a.offsets = offsets_dev;
    a.codes = codes_dev;
    a.ext_ids = ext_ids_dev;
    a.qcodes_out = qcodes_out_dev;
    a.ids = ids_dev;
    a.dists = dists_dev;
    a.part_i = part_i_dev;
    a.part_d = part_d_dev;
    a.split = split;
    a.dim = dim;
    a.k2 = k2;
    a.lmax = lmax;
    const int nbits = 8 * m;
    a.ht = ht > nbits ? nbits : ht;
    a.k = k;
    int cap = 512;  // room for the best k plus one step of 256 survivors
    while (cap < k + 256) cap <<= 1;
    a.cap = cap;
    a.direct = direct ? 1 : 0;
    const size_t lds = (size_t)2 * m * 256 * 4 + (size_t)dim * 4 + (size_t)cap * 8;  // (dim = 2 * m * ..: a multiple of 8 bytes)
    PSC_REQUIRE(lds <= 96 * 1024, "dimension and k too large for the multi-index scan");
    if (m == 8) {
        hipLaunchKernelGGL(imi_scan_kernel<8>, dim3((unsigned)(nq * split)), dim3(256), lds, s, a);
    } else {
        static bool configured = false;
        if (!configured) {
            PSC_HIP_TRY(hipFuncSetAttribute((const void *)imi_scan_kernel<16>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                            96 * 1024));
            configured = true;
        }
        hipLaunchKernelGGL(imi_scan_kernel<16>, dim3((unsigned)(nq * split)), dim3(256), lds, s, a);
    }
    PSC_HIP_TRY(hipGetLastError());
    char text[96];
    snprintf(text, sizeof text, "imi_scan_kernel%s m=%d cells<=%d pool=%d queries=%lld x%d", direct ? "+direct-tables" : "", m,
             lmax, cap, (long long)nq, split);
    note_scan_route(text);
    if (split > 1) return merge_partial_lists(part_d_dev, part_i_dev, nq, split, k, status_dev, ids_dev, dists_dev, s);
    return PSC_OK;
}

}  // namespace psc
