// Inverted-file variant (Section 2 "Non-exhaustive search", Section 4.3): coarse quantizer,
// selection of the lists to probe, and the device-side bookkeeping that turns the
// (query, probed list) jobs into list-major tiles for the fused scan.
//
// A query probes the nprobe coarse centroids nearest to it (squared L2 in float32, lower list
// number on equal distance; the three distance kernels -- plain, a handful of rows, matrix cores
// -- add the coordinates up in different orders, so they can rank two centroids that are equally
// near within float32 rounding differently).  Jobs are then grouped by list so
// that the codes of a list are streamed once per tile of up to TQ queries that probe it.
#include "common.h"

namespace psc {
namespace {

constexpr int kRows = 16;  // rows per workgroup in the distance kernels
// Up to this many rows (queries) the coarse stage runs the kernels built for latency: many
// workgroups per row instead of many rows per workgroup (from 256 rows the distances come from the
// matrix-core kernel where it is built for the dimension; the selection keeps a workgroup per row).
constexpr int64_t kFewRowsMax = 512;

// dist[r][c] = || x_r - cent_c ||^2 for a tile of kRows rows and 256 centroids per workgroup.
// Rows sit in LDS (read as broadcasts), each thread walks its own centroid row.
__global__ void __launch_bounds__(256)
coarse_dist_kernel(const float *__restrict__ x, int64_t n, int dim, const float *__restrict__ cent,
                   int nlist, float *__restrict__ dist)
{
    extern __shared__ __align__(16) float rows[];  // [kRows][dim]
    const int64_t r0 = (int64_t)blockIdx.x * kRows;
    for (int e = threadIdx.x; e < kRows * dim; e += 256) {
        const int64_t r = r0 + e / dim;
        rows[e] = r < n ? x[r * dim + e % dim] : 0.f;
    }
    __syncthreads();
    const int c = blockIdx.y * 256 + threadIdx.x;
    if (c >= nlist) return;
    const float *crow = cent + (int64_t)c * dim;
    float acc[kRows];
#pragma unroll
    for (int r = 0; r < kRows; ++r) acc[r] = 0.f;
    for (int d = 0; d < dim; d += 4) {
        const float4 cv = *(const float4 *)(crow + d);
#pragma unroll
        for (int r = 0; r < kRows; ++r) {
            const float4 xv = *(const float4 *)(rows + r * dim + d);
            float t = xv.x - cv.x;
            acc[r] = fmaf(t, t, acc[r]);
            t = xv.y - cv.y;
            acc[r] = fmaf(t, t, acc[r]);
            t = xv.z - cv.z;
            acc[r] = fmaf(t, t, acc[r]);
            t = xv.w - cv.w;
            acc[r] = fmaf(t, t, acc[r]);
        }
    }
#pragma unroll
    for (int r = 0; r < kRows; ++r)
        if (r0 + r < n) dist[(r0 + r) * nlist + c] = acc[r];
}

// The same distances for a handful of rows (a single query is the case that matters): one
// workgroup = 32 centroids x up to kFewRows rows, 8 lanes to a centroid, each lane taking every
// eighth group of 4 coordinates, so that the centroid rows are read in 128-byte pieces by many
// workgroups at once instead of one row per thread.  The 8 partial sums are added pairwise, so a
// distance can differ from coarse_dist_kernel's in its last bits.
constexpr int kFewRows = 4;

__global__ void __launch_bounds__(256)
coarse_dist_few_kernel(const float *__restrict__ x, int64_t n, int dim, const float *__restrict__ cent,
                       int nlist, float *__restrict__ dist)
{
    extern __shared__ __align__(16) float rows[];  // [kFewRows][dim]
    const int64_t r0 = (int64_t)blockIdx.y * kFewRows;
    for (int e = threadIdx.x; e < kFewRows * dim; e += 256) {
        const int64_t r = r0 + e / dim;
        rows[e] = r < n ? x[r * dim + e % dim] : 0.f;
    }
    __syncthreads();
    const int sub = threadIdx.x & 7;
    const int c = blockIdx.x * 32 + (threadIdx.x >> 3);
    float acc[kFewRows];
#pragma unroll
    for (int r = 0; r < kFewRows; ++r) acc[r] = 0.f;
    if (c < nlist) {
        const float *crow = cent + (int64_t)c * dim;
        for (int d = sub * 4; d < dim; d += 32) {
            const float4 cv = *(const float4 *)(crow + d);
#pragma unroll
            for (int r = 0; r < kFewRows; ++r) {
                const float4 xv = *(const float4 *)(rows + r * dim + d);
                float t = xv.x - cv.x;
                acc[r] = fmaf(t, t, acc[r]);
                t = xv.y - cv.y;
                acc[r] = fmaf(t, t, acc[r]);
                t = xv.z - cv.z;
                acc[r] = fmaf(t, t, acc[r]);
                t = xv.w - cv.w;
                acc[r] = fmaf(t, t, acc[r]);
            }
        }
    }
#pragma unroll
    for (int r = 0; r < kFewRows; ++r) {
        acc[r] += __shfl_xor(acc[r], 1, 64);
        acc[r] += __shfl_xor(acc[r], 2, 64);
        acc[r] += __shfl_xor(acc[r], 4, 64);
        if (sub == 0 && c < nlist && r0 + r < n) dist[(r0 + r) * nlist + c] = acc[r];
    }
}

__device__ __forceinline__ uint64_t order_key(float d, uint32_t idx)
{
    const uint32_t u = __float_as_uint(d + 0.0f);
    const uint32_t key = u ^ ((uint32_t)((int32_t)u >> 31) | 0x80000000u);
    return ((uint64_t)key << 32) | idx;
}

__device__ __forceinline__ uint64_t wave_min_u64(uint64_t v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const uint64_t o = __shfl_xor(v, off, 64);
        v = o < v ? o : v;
    }
    return v;
}

// Sum of v over the wave, in every lane (row-local steps on the data-parallel path, the four row
// sums through scalar registers).
__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v)
{
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xf, 0xf, false);   // lane ^ 1
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xf, 0xf, false);   // lane ^ 2
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xf, 0xf, false);  // mirror in 8
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xf, 0xf, false);  // mirror in 16
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 0) + (uint32_t)__builtin_amdgcn_readlane((int)v, 16) +
           (uint32_t)__builtin_amdgcn_readlane((int)v, 32) + (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
}

// The nprobe nearest lists of a row, one wave per row, the row's nlist <= 64 KPL distance keys
// in registers (lane l holds lists l, l + 64, ...).
//  1. the nprobe-th smallest distance key, bit by bit: a bit of the answer is 0 iff at least
//     nprobe keys lie below (the bits found so far, this bit set);
//  2. selected = keys below it, plus the lowest-numbered lists among the keys equal to it;
//  3. the selected (key, list) pairs go to LDS and every one is written to its rank.
template <int KPL>
__global__ void __launch_bounds__(256)
select_probes_wave_kernel(const float *__restrict__ dist, int64_t n, int nlist, int nprobe,
                          const int32_t *__restrict__ settled, int32_t *__restrict__ probed)
{
    extern __shared__ __align__(16) uint64_t sel[];  // [4][nprobe]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t r = (int64_t)blockIdx.x * 4 + wave;
    if (r >= n) return;
    if (settled && settled[r] >= 0) return;  // (the waves of a workgroup meet at no barrier)
    uint64_t *mine = sel + (size_t)wave * nprobe;
    uint32_t dk[KPL];
#pragma unroll
    for (int i = 0; i < KPL; ++i) {
        const int c = i * 64 + lane;
        // (real keys stay below the filler of the places past the last list, whatever the distance)
        dk[i] = c < nlist ? min((uint32_t)(order_key(dist[r * nlist + c], 0u) >> 32), 0xfffffffeu) : 0xffffffffu;
    }
    uint32_t pivot = 0;
    for (int b = 31; b >= 0; --b) {
        const uint32_t mid = pivot | (1u << b);
        uint32_t cnt = 0;
#pragma unroll
        for (int i = 0; i < KPL; ++i) cnt += dk[i] < mid ? 1u : 0u;
        if (wave_sum_u32(cnt) < (uint32_t)nprobe) pivot = mid;
    }
    uint32_t below = 0;
#pragma unroll
    for (int i = 0; i < KPL; ++i) below += dk[i] < pivot ? 1u : 0u;
    int take = nprobe - (int)wave_sum_u32(below);  // how many of the keys equal to the pivot belong
    int at = 0;                                     // selected so far
#pragma unroll
    for (int i = 0; i < KPL; ++i) {
        const bool eq = dk[i] == pivot;
        const uint64_t eqm = __ballot(eq);
        const int before = __builtin_popcountll(eqm & ((1ull << lane) - 1ull));
        const bool chosen = dk[i] < pivot || (eq && before < take);
        take -= __builtin_popcountll(eqm);
        const uint64_t cm = __ballot(chosen);
        if (chosen) mine[at + __builtin_popcountll(cm & ((1ull << lane) - 1ull))] = ((uint64_t)dk[i] << 32) | (uint32_t)(i * 64 + lane);
        at += __builtin_popcountll(cm);
    }
    __builtin_amdgcn_wave_barrier();
    for (int e = lane; e < nprobe; e += 64) {
        const uint64_t key = mine[e];
        int rank = 0;
        for (int j = 0; j < nprobe; ++j) rank += mine[j] < key ? 1 : 0;
        probed[r * nprobe + rank] = (int32_t)(uint32_t)key;
    }
}

// The same selection by a whole workgroup of 16 waves per row, for a handful of rows (a single
// query is the case that matters): thread t holds lists t, t + 1024, ...  The nprobe-th smallest
// (distance, list) pair is found bit by bit as above -- first over the 32 bits of the distance
// key, then, only if several lists share that distance, over the 14 bits of the list number --
// with one workgroup-wide count per bit (per-wave sums through LDS, two buffers in turn so that
// one barrier per bit is enough).  The pairs up to it are exactly the nprobe lists; each goes to
// its rank.
template <int KPL>
__global__ void __launch_bounds__(1024)
select_probes_block_kernel(const float *__restrict__ dist, int nlist, int nprobe, const int32_t *__restrict__ settled,
                           int32_t *__restrict__ probed)
{
    __shared__ uint32_t part[2][16];
    __shared__ uint64_t sel[1024];
    __shared__ uint32_t nsel;
    const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t r = blockIdx.x;
    if (settled && settled[r] >= 0) return;  // (the whole workgroup: one row)
    uint32_t dk[KPL];
#pragma unroll
    for (int i = 0; i < KPL; ++i) {
        const int c = i * 1024 + tid;
        dk[i] = c < nlist ? min((uint32_t)(order_key(dist[r * nlist + c], 0u) >> 32), 0xfffffffeu) : 0xffffffffu;
    }
    if (tid == 0) nsel = 0u;
    int turn = 0;
    // number of keys for which `below(i)` holds, over the whole workgroup
    auto count = [&](auto below) {
        uint32_t cnt = 0;
#pragma unroll
        for (int i = 0; i < KPL; ++i) cnt += below(i) ? 1u : 0u;
        cnt = wave_sum_u32(cnt);
        if (lane == 0) part[turn][wave] = cnt;
        __syncthreads();
        uint32_t total = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) total += part[turn][w];
        turn ^= 1;
        return total;
    };
    uint32_t pivot = 0;
    for (int b = 31; b >= 0; --b) {
        const uint32_t mid = pivot | (1u << b);
        if (count([&](int i) { return dk[i] < mid; }) < (uint32_t)nprobe) pivot = mid;
    }
    // lists at the pivot distance: all of them belong unless they are too many; then the
    // lowest-numbered ones do, up to list number `last`
    const uint32_t below = count([&](int i) { return dk[i] < pivot; });
    const uint32_t upto = count([&](int i) { return dk[i] <= pivot; });
    uint32_t last = 0xffffffffu;
    if (upto > (uint32_t)nprobe) {
        const uint32_t want = (uint32_t)nprobe - below;  // >= 1
        uint32_t lp = 0;
        for (int b = 13; b >= 0; --b) {
            const uint32_t mid = lp | (1u << b);
            if (count([&](int i) { return dk[i] == pivot && (uint32_t)(i * 1024 + tid) < mid; }) < want) lp = mid;
        }
        last = lp;
    }
#pragma unroll
    for (int i = 0; i < KPL; ++i) {
        const uint32_t c = (uint32_t)(i * 1024 + tid);
        if (dk[i] < pivot || (dk[i] == pivot && c <= last)) {
            const uint32_t slot = atomicAdd(&nsel, 1u);
            if (slot < 1024u) sel[slot] = ((uint64_t)dk[i] << 32) | c;  // (exactly nprobe <= 1024 pass)
        }
    }
    __syncthreads();
    if (tid < nprobe) {
        const uint64_t key = sel[tid];
        int rank = 0;
        for (int j = 0; j < nprobe; ++j) rank += sel[j] < key ? 1 : 0;
        probed[r * nprobe + rank] = (int32_t)(uint32_t)key;
    }
}

// More than 4096 lists.  One workgroup per row: nprobe times take the smallest remaining
// (distance, list) key.
__global__ void __launch_bounds__(256)
select_probes_kernel(const float *__restrict__ dist, int nlist, int nprobe, const int32_t *__restrict__ settled,
                     int32_t *__restrict__ probed)
{
    extern __shared__ __align__(16) uint64_t keys[];  // [nlist]
    __shared__ uint64_t wave_best[4];
    const int64_t r = blockIdx.x;
    if (settled && settled[r] >= 0) return;  // (the whole workgroup: one row)
    for (int c = threadIdx.x; c < nlist; c += 256) keys[c] = order_key(dist[r * nlist + c], (uint32_t)c);
    __syncthreads();
    for (int p = 0; p < nprobe; ++p) {
        uint64_t best = ~0ull;
        for (int c = threadIdx.x; c < nlist; c += 256) {
            const uint64_t v = keys[c];
            best = v < best ? v : best;
        }
        best = wave_min_u64(best);
        if ((threadIdx.x & 63) == 0) wave_best[threadIdx.x >> 6] = best;
        __syncthreads();
        uint64_t b = wave_best[0];
#pragma unroll
        for (int w = 1; w < 4; ++w) b = wave_best[w] < b ? wave_best[w] : b;
        const uint32_t sel = (uint32_t)b;
        if (threadIdx.x == 0) {
            probed[r * nprobe + p] = (int32_t)sel;
            keys[sel] = ~0ull;
        }
        __syncthreads();
    }
}

// Nearest centroid per row: the same distance arithmetic as coarse_dist_kernel, with a running
// (distance, number) minimum per thread over all centroid blocks and one reduction per row.
__global__ void __launch_bounds__(256)
nearest_centroid_kernel(const float *__restrict__ x, int64_t n, int dim, const float *__restrict__ cent,
                        int nlist, int32_t *__restrict__ assign)
{
    extern __shared__ __align__(16) float rows[];  // [kRows][dim], then 4*kRows uint64 for the reduction
    const int64_t r0 = (int64_t)blockIdx.x * kRows;
    for (int e = threadIdx.x; e < kRows * dim; e += 256) {
        const int64_t r = r0 + e / dim;
        rows[e] = r < n ? x[r * dim + e % dim] : 0.f;
    }
    __syncthreads();
    uint64_t best[kRows];
#pragma unroll
    for (int r = 0; r < kRows; ++r) best[r] = ~0ull;
    for (int c = threadIdx.x; c < nlist; c += 256) {
        const float *crow = cent + (int64_t)c * dim;
        float acc[kRows];
#pragma unroll
        for (int r = 0; r < kRows; ++r) acc[r] = 0.f;
        for (int d = 0; d < dim; d += 4) {
            const float4 cv = *(const float4 *)(crow + d);
#pragma unroll
            for (int r = 0; r < kRows; ++r) {
                const float4 xv = *(const float4 *)(rows + r * dim + d);
                float t = xv.x - cv.x;
                acc[r] = fmaf(t, t, acc[r]);
                t = xv.y - cv.y;
                acc[r] = fmaf(t, t, acc[r]);
                t = xv.z - cv.z;
                acc[r] = fmaf(t, t, acc[r]);
                t = xv.w - cv.w;
                acc[r] = fmaf(t, t, acc[r]);
            }
        }
#pragma unroll
        for (int r = 0; r < kRows; ++r) {
            const uint64_t key = order_key(acc[r], (uint32_t)c);
            best[r] = key < best[r] ? key : best[r];
        }
    }
    __syncthreads();  // rows no longer needed: reuse LDS for the cross-wave reduction
    uint64_t *red = (uint64_t *)rows;
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
        const uint64_t b = wave_min_u64(best[r]);
        if ((threadIdx.x & 63) == 0) red[(threadIdx.x >> 6) * kRows + r] = b;
    }
    __syncthreads();
    if (threadIdx.x < kRows && r0 + threadIdx.x < n) {
        uint64_t b = red[threadIdx.x];
        for (int w = 1; w < 4; ++w) b = red[w * kRows + threadIdx.x] < b ? red[w * kRows + threadIdx.x] : b;
        assign[r0 + threadIdx.x] = (int32_t)(uint32_t)b;
    }
}

// ---------------------------------------------------------------------------------------------
// Nearest centroid on the matrix cores (the assignment step of Section 4.3's index, and of the
// coarse k-means): arg-min over c of || x - c ||^2 = arg-min of || c' ||^2 - 2 x'.c' with
// x' = x - mu, c' = c - mu (mu: any common reference point, here the mean centroid; centring keeps
// the terms small and with them the rounding error of the expansion, about 1e-7 of the distance).
// The cross term is a dense [rows x DIM] . [DIM x nlist] contraction in full float32
// (v_mfma_f32_32x32x2f32, operand layout as in the table kernel: A[i][k] with i = lane % 32,
// k = lane / 32; D[i][j] in 16 registers, register v = row 8 * (v / 4) + 4 * (lane / 32) + v % 4,
// column j = lane % 32).
// One workgroup = 4 waves x 32 rows; the rows sit in registers for the whole kernel (DIM / 2 per
// lane), the centroids stream through LDS in tiles of 32 (double-buffered, centred and their
// norms taken while staging), and every lane keeps the running minimum of its 16 outputs.  Ties
// go to the lower centroid number, as in the plain kernel; the two kernels can differ where two
// centroids are equally near within float32 rounding.
// ---------------------------------------------------------------------------------------------
typedef float f32x16 __attribute__((ext_vector_type(16)));

// DIST: instead of the arg-min, all distances || x - c ||^2 = || x' ||^2 + || c' ||^2 - 2 x'.c' are
// written (dist [n][nlist], clamped at 0), and the grid's second dimension splits the centroid
// tiles into groups of kDistTilesPerGroup so that a small batch of rows still fills the chip.
constexpr int kDistTilesPerGroup = 8;

template <int DIM, bool DIST>
__global__ void __launch_bounds__(256)
nearest_centroid_mfma_kernel(const float *__restrict__ x, int64_t n, const float *__restrict__ cent,
                             const float *__restrict__ mu, int nlist, int32_t *__restrict__ assign,
                             float *__restrict__ dist)
{
    static_assert(DIM % 8 == 0 && DIM <= 128, "rows are held in registers");
    constexpr int KS = DIM / 2;
    constexpr int LD = DIM + 2;  // row pitch of a staged tile: lanes (half, col) hit 64 different banks
    __shared__ float tile[2][32 * LD];
    __shared__ float cnorm[2][32];
    __shared__ float xnorm[4][32];
    const int tid = (int)threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int half = lane >> 5, col = lane & 31;
    const int64_t r0 = (int64_t)blockIdx.x * 128 + wave * 32;

    float a[KS];
    {
        const int64_t r = r0 + col;
        const float *xr = x + (r < n ? r : n - 1) * DIM;
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) a[kk] = xr[2 * kk + half] - mu[2 * kk + half];
    }
    if constexpr (DIST) {  // || x' ||^2 of row `col`: this lane's coordinates plus the other half's
        float xn = 0.f;
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) xn = fmaf(a[kk], a[kk], xn);
        xn += __shfl_xor(xn, 32, 64);
        if (half == 0) xnorm[wave][col] = xn;
        __builtin_amdgcn_wave_barrier();
    }
    // staging: thread -> centroid tid / 8 of the tile, coordinates (tid % 8) * 4 + 32 * i
    const int sc = tid >> 3, sp = (tid & 7) * 4;
    auto stage = [&](int t, int buf) {
        const int c = t * 32 + sc;
        float nrm = 0.f;
#pragma unroll
        for (int i = 0; i < DIM / 32; ++i) {
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (c < nlist) {
                v = *(const float4 *)(cent + (int64_t)c * DIM + sp + 32 * i);
                const float4 m = *(const float4 *)(mu + sp + 32 * i);
                v.x -= m.x;
                v.y -= m.y;
                v.z -= m.z;
                v.w -= m.w;
            }
            float *d = &tile[buf][sc * LD + sp + 32 * i];
            d[0] = v.x;
            d[1] = v.y;
            d[2] = v.z;
            d[3] = v.w;
            nrm = fmaf(v.x, v.x, nrm);
            nrm = fmaf(v.y, v.y, nrm);
            nrm = fmaf(v.z, v.z, nrm);
            nrm = fmaf(v.w, v.w, nrm);
        }
        nrm += __shfl_xor(nrm, 1, 64);
        nrm += __shfl_xor(nrm, 2, 64);
        nrm += __shfl_xor(nrm, 4, 64);
        if ((tid & 7) == 0) cnorm[buf][sc] = c < nlist ? nrm : __builtin_inff();
    };
    float bestv[16];
    int besti[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        bestv[v] = __builtin_inff();
        besti[v] = 0;
    }
    const int tiles_all = (nlist + 31) / 32;
    const int tbeg = DIST ? (int)blockIdx.y * kDistTilesPerGroup : 0;
    const int ntiles = DIST ? (tiles_all < tbeg + kDistTilesPerGroup ? tiles_all : tbeg + kDistTilesPerGroup) : tiles_all;
    stage(tbeg, tbeg & 1);
    __syncthreads();
    for (int t = tbeg; t < ntiles; ++t) {
        const int buf = t & 1;
        if (t + 1 < ntiles) stage(t + 1, buf ^ 1);
        f32x16 acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.f;
        const float *b = &tile[buf][col * LD + half];
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[kk], b[2 * kk], acc, 0, 0, 0);
        const float cn = cnorm[buf][col];
        const int ci = t * 32 + col;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const float d = fmaf(-2.0f, acc[v], cn);  // (+inf for the padding of the last tile)
            if constexpr (DIST) {
                const int i = 8 * (v / 4) + 4 * half + v % 4;
                if (r0 + i < n && ci < nlist) {
                    const float full = d + xnorm[wave][i];
                    dist[(r0 + i) * nlist + ci] = full > 0.f ? full : 0.f;
                }
            } else if (d < bestv[v]) {
                bestv[v] = d;
                besti[v] = ci;
            }
        }
        __syncthreads();
    }
    if constexpr (DIST) return;
    // the 32 lanes of a half hold the 32 columns of each of its 16 rows: smallest (value, number)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        float bv = bestv[v];
        int bi = besti[v];
#pragma unroll
        for (int off = 16; off >= 1; off >>= 1) {
            const float ov = __shfl_xor(bv, off, 64);
            const int oi = __shfl_xor(bi, off, 64);
            if (ov < bv || (ov == bv && oi < bi)) {
                bv = ov;
                bi = oi;
            }
        }
        const int64_t r = r0 + 8 * (v / 4) + 4 * half + v % 4;
        if (col == 0 && r < n) assign[r] = bi;
    }
}

// ---------------------------------------------------------------------------------------------
// Job bookkeeping.  Jobs in query-major order are cut into blocks of kJobBlockQ queries; a
// stable counting sort by list number (block histograms -> column prefix -> in-order scatter)
// gives every list its jobs in ascending query order, reproducibly.
// ---------------------------------------------------------------------------------------------
constexpr int kJobBlockQ = 16;

__global__ void zero_i32_kernel(int32_t *p, int64_t n)
{
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e < n) p[e] = 0;
}

// Sort key of job (q, p): its list, with the jobs of a query's `pilot` nearest lists ahead of all
// others (keys [0, nlist) before keys [nlist, 2 nlist)).  Workgroups start in tile order, so the
// nearest lists of every query are scanned first and their k-th best distances are published
// before the bulk of the lists is looked at, which then rejects most survivors at the threshold
// test instead of inserting them into lists.
__device__ __forceinline__ int job_key(int list, int p, int nlist, int pilot) { return list + (p >= pilot ? nlist : 0); }

__global__ void job_hist_kernel(const int32_t *__restrict__ probed, int64_t nq, int nprobe, int nlist, int pilot,
                                int32_t *__restrict__ hist)
{
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= nq * nprobe) return;
    const int64_t q = j / nprobe;
    const int p = (int)(j - q * nprobe);
    atomicAdd(&hist[(q / kJobBlockQ) * (2 * nlist) + job_key(probed[j], p, nlist, pilot)], 1);
}

// hist[b][l] -> number of jobs of list l in blocks before b; totals[l] = jobs of list l.
__global__ void job_column_prefix_kernel(int32_t *__restrict__ hist, int64_t nblk, int nlist,
                                         int32_t *__restrict__ totals)
{
    const int l = blockIdx.x * blockDim.x + threadIdx.x;
    if (l >= nlist) return;
    int32_t run = 0;
    int64_t b = 0;
    for (; b + 16 <= nblk; b += 16) {  // sixteen loads in flight instead of one (the walk is latency-bound)
        int32_t c[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) c[i] = hist[(b + i) * nlist + l];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            hist[(b + i) * nlist + l] = run;
            run += c[i];
        }
    }
    for (; b < nblk; ++b) {
        const int32_t c = hist[b * nlist + l];
        hist[b * nlist + l] = run;
        run += c;
    }
    totals[l] = run;
}

// One workgroup: list_begin = exclusive prefix of totals; tile_begin = exclusive prefix of
// ceil(totals / tq).  `totals` aliases list_begin (read before written, element-wise by owner).
__global__ void __launch_bounds__(1024)
job_list_prefix_kernel(int32_t *__restrict__ list_begin, int32_t *__restrict__ tile_begin, int nlist, int tq)
{
    __shared__ int32_t pj[1024], pt[1024];
    const int t = threadIdx.x;
    const int per = (nlist + 1023) / 1024;
    const int lo = t * per, hi = min(nlist, lo + per);
    int32_t sj = 0, st = 0;
    for (int l = lo; l < hi; ++l) {
        sj += list_begin[l];
        st += (list_begin[l] + tq - 1) / tq;
    }
    pj[t] = sj;
    pt[t] = st;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {
        const int32_t aj = t >= off ? pj[t - off] : 0, at = t >= off ? pt[t - off] : 0;
        __syncthreads();
        pj[t] += aj;
        pt[t] += at;
        __syncthreads();
    }
    int32_t bj = pj[t] - sj, bt = pt[t] - st;  // exclusive
    for (int l = lo; l < hi; ++l) {
        const int32_t c = list_begin[l];
        list_begin[l] = bj;
        tile_begin[l] = bt;
        bj += c;
        bt += (c + tq - 1) / tq;
    }
    if (t == 1023) {
        list_begin[nlist] = pj[1023];
        tile_begin[nlist] = pt[1023];
    }
}

// One workgroup per block of kJobBlockQ queries, queries taken in order: job (q, p) goes to
// list_begin[l] + (jobs of l in earlier blocks) + (jobs of l earlier in this block).
__global__ void __launch_bounds__(256)
job_scatter_kernel(const int32_t *__restrict__ probed, int64_t nq, int nprobe, int nlist, int pilot,
                   int32_t *__restrict__ hist, const int32_t *__restrict__ list_begin,
                   int32_t *__restrict__ job_q, int32_t *__restrict__ job_list, int32_t *__restrict__ job_slot)
{
    const int64_t b = blockIdx.x;
    int32_t *run = hist + b * (2 * nlist);
    for (int qi = 0; qi < kJobBlockQ; ++qi) {
        const int64_t q = b * kJobBlockQ + qi;
        if (q >= nq) break;
        for (int p = threadIdx.x; p < nprobe; p += 256) {  // the lists of one query are distinct
            const int l = probed[q * nprobe + p];
            const int key = job_key(l, p, nlist, pilot);
            // the only writer of run[key] in this turn; the atomic keeps it coherent across turns
            const int32_t at = list_begin[key] + atomicAdd(&run[key], 1);
            job_q[at] = (int32_t)q;
            job_list[at] = l;
            job_slot[at] = (int32_t)(q * nprobe + p);
        }
        __syncthreads();
    }
}

struct TileRec {
    int32_t job_begin, njobs, list, pad;
};

__global__ void job_tiles_kernel(const int32_t *__restrict__ list_begin, const int32_t *__restrict__ tile_begin,
                                 int nlist, int tq, TileRec *__restrict__ tiles)
{
    const int key = blockIdx.x * blockDim.x + threadIdx.x;
    if (key >= 2 * nlist) return;
    const int l = key < nlist ? key : key - nlist;
    const int32_t jb = list_begin[key], cnt = list_begin[key + 1] - jb;
    int32_t t = tile_begin[key];
    for (int32_t o = 0; o < cnt; o += tq, ++t) tiles[t] = TileRec{jb + o, min(tq, cnt - o), l, 0};
}

// Few jobs: no grouping by list.  Every job becomes a tile of its own, the jobs of every query's
// nearest list first, then all second nearest, ...: tile t = (query t % nq, probe t / nq).
__global__ void direct_jobs_kernel(const int32_t *__restrict__ probed, int nq, int nprobe,
                                   int32_t *__restrict__ job_q, int32_t *__restrict__ job_list,
                                   int32_t *__restrict__ job_slot, TileRec *__restrict__ tiles,
                                   int32_t *__restrict__ ntiles)
{
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    const int njobs = nq * nprobe;
    if (t == 0) *ntiles = njobs;
    if (t >= njobs) return;
    const int p = t / nq, q = t - p * nq;
    const int l = probed[q * nprobe + p];
    job_q[t] = q;
    job_list[t] = l;
    job_slot[t] = q * nprobe + p;
    tiles[t] = TileRec{t, 1, l, 0};
}

// The lists' share of the residual tables: see launch_list_tables.  One workgroup per (list,
// sub-quantizer), thread c owns centroid c.
__global__ void __launch_bounds__(256)
list_tables_kernel(const float *__restrict__ cb, int dim, int m, const float *__restrict__ coarse, int nlist,
                   float *__restrict__ out)
{
    extern __shared__ float gt[];  // (g_l - o)_j
    const int l = blockIdx.x, j = blockIdx.y, c = threadIdx.x;
    const int dsub = dim / m;
    for (int t = threadIdx.x; t < dsub; t += 256)
        gt[t] = coarse[(int64_t)l * dim + j * dsub + t] - coarse[(int64_t)nlist * dim + j * dsub + t];
    __syncthreads();
    const float *crow = cb + ((int64_t)j * 256 + c) * dsub;
    float acc = 0.f;
    for (int t = 0; t < dsub; ++t) acc = fmaf(gt[t], crow[t], acc);
    out[((int64_t)l * m + j) * 256 + c] = 2.0f * acc;
}

// Copy per-job rows (job-sorted) back to (query, probe) order.
__global__ void unsort_rows_kernel(const uint8_t *__restrict__ src, const int32_t *__restrict__ job_slot,
                                   int64_t njobs, int row_bytes, uint8_t *__restrict__ dst)
{
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= njobs * row_bytes) return;
    const int64_t j = e / row_bytes;
    dst[(int64_t)job_slot[j] * row_bytes + e % row_bytes] = src[e];
}

}  // namespace

int launch_list_tables(const float *cb_dev, int dim, int m, const float *coarse_dev, int nlist,
                       float *list_tab_dev, hipStream_t s)
{
    PSC_REQUIRE(dim % m == 0 && nlist >= 1, "bad shape");
    hipLaunchKernelGGL(list_tables_kernel, dim3((unsigned)nlist, (unsigned)m), dim3(256),
                       (size_t)(dim / m) * sizeof(float), s, cb_dev, dim, m, coarse_dev, nlist, list_tab_dev);
    PSC_HIP_TRY(hipGetLastError());
    return PSC_OK;
}

int launch_unsort_rows(const uint8_t *src_dev, const int32_t *job_slot_dev, int64_t njobs, int row_bytes,
                       uint8_t *dst_dev, hipStream_t s)
{
    const int64_t total = njobs * row_bytes;
    if (total == 0) return PSC_OK;
    hipLaunchKernelGGL(unsort_rows_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, src_dev,
                       job_slot_dev, njobs, row_bytes, dst_dev);
    PSC_HIP_TRY(hipGetLastError());
    return PSC_OK;
}

static int check_dim(int dim, int nlist)
{
    PSC_REQUIRE(dim > 0 && dim % 4 == 0 && dim <= 1024, "coarse quantizer needs dim %% 4 == 0 and dim <= 1024, got %d", dim);
    PSC_REQUIRE(nlist >= 1 && nlist <= 16384, "nlist must be in [1, 16384], got %d", nlist);
    return PSC_OK;
}

template <int DIM>
static int run_coarse_dist_mfma(const float *x_dev, int64_t n, const float *cent_dev, const float *mu_dev, int nlist,
                                float *dist_dev, hipStream_t s)
{
    const int tiles = (nlist + 31) / 32;
    dim3 grid((unsigned)((n + 127) / 128), (unsigned)((tiles + kDistTilesPerGroup - 1) / kDistTilesPerGroup));
    hipLaunchKernelGGL((nearest_centroid_mfma_kernel<DIM, true>), grid, dim3(256), 0, s, x_dev, n, cent_dev, mu_dev,
                       nlist, (int32_t *)nullptr, dist_dev);
    PSC_HIP_TRY(hipGetLastError());
    return PSC_OK;
}

// mu_dev: reference point [dim] of the matrix-core kernel (the mean centroid), which takes batches
// of 256 rows and more in the dimensions it is built for; everything else takes the plain kernel.
int launch_coarse_distances(const float *x_dev, int64_t n, int dim, const float *cent_dev, int nlist,
                            const float *mu_dev, float *dist_dev, hipStream_t s)
{
    int rc = check_dim(dim, nlist);
    if (rc != PSC_OK) return rc;
    if (n == 0) return PSC_OK;
    if (mu_dev && n >= 256 && (n + 127) / 128 <= 0x7fffffffLL) {
        switch (dim) {
        case 32: return run_coarse_dist_mfma<32>(x_dev, n, cent_dev, mu_dev, nlist, dist_dev, s);
        case 64: return run_coarse_dist_mfma<64>(x_dev, n, cent_dev, mu_dev, nlist, dist_dev, s);
        case 96: return run_coarse_dist_mfma<96>(x_dev, n, cent_dev, mu_dev, nlist, dist_dev, s);
        case 128: return run_coarse_dist_mfma<128>(x_dev, n, cent_dev, mu_dev, nlist, dist_dev, s);
        default: break;
        }
    }
    if (n <= kFewRowsMax) {
        dim3 grid((unsigned)((nlist + 31) / 32), (unsigned)((n + kFewRows - 1) / kFewRows));
        hipLaunchKernelGGL(coarse_dist_few_kernel, grid, dim3(256), (size_t)kFewRows * dim * sizeof(float), s, x_dev, n,
                           dim, cent_dev, nlist, dist_dev);
        PSC_HIP_TRY(hipGetLastError());
        return PSC_OK;
    }
    PSC_REQUIRE((n + kRows - 1) / kRows <= 0x7fffffffLL, "too many rows");
    dim3 grid((unsigned)((n + kRows - 1) / kRows), (unsigned)((nlist + 255) / 256));
    hipLaunchKernelGGL(coarse_dist_kernel, grid, dim3(256), (size_t)kRows * dim * sizeof(float), s, x_dev, n, dim,
                       cent_dev, nlist, dist_dev);
    PSC_HIP_TRY(hipGetLastError());
    return PSC_OK;
}

int launch_select_probes(const float *dist_dev, int64_t n, int nlist, int nprobe, const int32_t *settled_dev,
                         int32_t *probed_dev, hipStream_t s)
{
    PSC_REQUIRE(nprobe >= 1 && nprobe <= nlist && nlist <= 16384, "bad nprobe/nlist");
    if (n == 0) return PSC_OK;
    PSC_REQUIRE(n <= 0x7fffffffLL, "too many rows");
    static bool configured = false;
    if (!configured) {
        PSC_HIP_TRY(hipFuncSetAttribute((const void *)select_probes_kernel,
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 16384 * 8));
        configured = true;
    }
    if (n <= kFewRowsMax) {  // a workgroup per row: the latency of a single query
        if (nlist <= 4096)
            hipLaunchKernelGGL(select_probes_block_kernel<4>, dim3((unsigned)n), dim3(1024), 0, s, dist_dev, nlist,
                               nprobe, settled_dev, probed_dev);
        else
            hipLaunchKernelGGL(select_probes_block_kernel<16>, dim3((unsigned)n), dim3(1024), 0, s, dist_dev, nlist,
                               nprobe, settled_dev, probed_dev);
        PSC_HIP_TRY(hipGetLastError());
        return PSC_OK;
    }
    const dim3 wgrid((unsigned)((n + 3) / 4));
    const size_t wlds = (size_t)4 * nprobe * sizeof(uint64_t);
    if (nlist <= 1024)
        hipLaunchKernelGGL(select_probes_wave_kernel<16>, wgrid, dim3(256), wlds, s, dist_dev, n, nlist, nprobe,
                           settled_dev, probed_dev);
    else if (nlist <= 4096)
        hipLaunchKernelGGL(select_probes_wave_kernel<64>, wgrid, dim3(256), wlds, s, dist_dev, n, nlist, nprobe,
                           settled_dev, probed_dev);
    else
        hipLaunchKernelGGL(select_probes_kernel, dim3((unsigned)n), dim3(256), (size_t)nlist * sizeof(uint64_t), s,
                           dist_dev, nlist, nprobe, settled_dev, probed_dev);
    PSC_HIP_TRY(hipGetLastError());
    return PSC_OK;
}

template <int DIM>
static int run_nearest_centroid_mfma(const float *x_dev, int64_t n, const float *cent_dev, const float *mu_dev,
                                     int nlist, int32_t *assign_dev, hipStream_t s)
{
    hipLaunchKernelGGL((nearest_centroid_mfma_kernel<DIM, false>), dim3((unsigned)((n + 127) / 128)), dim3(256), 0, s,
                       x_dev, n, cent_dev, mu_dev, nlist, assign_dev, (float *)nullptr);
    PSC_HIP_TRY(hipGetLastError());
    return PSC_OK;
}

// mu_dev: a reference point [dim] for the matrix-core kernel (the mean centroid); null, or a
// dimension that kernel is not built for, takes the plain kernel.
int launch_nearest_centroid(const float *x_dev, int64_t n, int dim, const float *cent_dev, int nlist,
                            const float *mu_dev, int32_t *assign_dev, hipStream_t s)
{
    int rc = check_dim(dim, nlist);
    if (rc != PSC_OK) return rc;
    if (n == 0) return PSC_OK;
    if (mu_dev && (n + 127) / 128 <= 0x7fffffffLL) {
        switch (dim) {
        case 32: return run_nearest_centroid_mfma<32>(x_dev, n, cent_dev, mu_dev, nlist, assign_dev, s);
        case 64: return run_nearest_centroid_mfma<64>(x_dev, n, cent_dev, mu_dev, nlist, assign_dev, s);
        case 96: return run_nearest_centroid_mfma<96>(x_dev, n, cent_dev, mu_dev, nlist, assign_dev, s);
        case 128: return run_nearest_centroid_mfma<128>(x_dev, n, cent_dev, mu_dev, nlist, assign_dev, s);
        default: break;
        }
    }
    PSC_REQUIRE((n + kRows - 1) / kRows <= 0x7fffffffLL, "too many rows");
    size_t lds = (size_t)kRows * dim * sizeof(float);
    if (lds < 4 * kRows * sizeof(uint64_t)) lds = 4 * kRows * sizeof(uint64_t);
    hipLaunchKernelGGL(nearest_centroid_kernel, dim3((unsigned)((n + kRows - 1) / kRows)), dim3(256), lds, s,
                       x_dev, n, dim, cent_dev, nlist, assign_dev);
    PSC_HIP_TRY(hipGetLastError());
    return PSC_OK;
}

int launch_build_jobs(const int32_t *probed_dev, int64_t nq, int nprobe, int nlist, int pilot, int tq,
                      const IvfJobBuffers &b, hipStream_t s)
{
    const int64_t njobs = nq * nprobe;
    if (njobs <= kDirectJobs) {  // a few queries: latency matters, sharing of code loads does not
        hipLaunchKernelGGL(direct_jobs_kernel, dim3((unsigned)((njobs + 255) / 256)), dim3(256), 0, s, probed_dev,
                           (int)nq, nprobe, b.job_q, b.job_list, b.job_slot, (TileRec *)b.tiles,
                           b.tile_begin + 2 * nlist);
        PSC_HIP_TRY(hipGetLastError());
        return PSC_OK;
    }
    const int64_t nblk = (nq + kJobBlockQ - 1) / kJobBlockQ;
    const int nkeys = 2 * nlist;
    PSC_REQUIRE(njobs < 0x7fffffffLL && nblk * nkeys < ((int64_t)1 << 40), "too many jobs");
    const int64_t hcells = nblk * nkeys;
    hipLaunchKernelGGL(zero_i32_kernel, dim3((unsigned)((hcells + 255) / 256)), dim3(256), 0, s, b.hist, hcells);
    hipLaunchKernelGGL(job_hist_kernel, dim3((unsigned)((njobs + 255) / 256)), dim3(256), 0, s, probed_dev, nq,
                       nprobe, nlist, pilot, b.hist);
    hipLaunchKernelGGL(job_column_prefix_kernel, dim3((unsigned)((nkeys + 255) / 256)), dim3(256), 0, s, b.hist,
                       nblk, nkeys, b.list_begin);
    hipLaunchKernelGGL(job_list_prefix_kernel, dim3(1), dim3(1024), 0, s, b.list_begin, b.tile_begin, nkeys, tq);
    hipLaunchKernelGGL(job_scatter_kernel, dim3((unsigned)nblk), dim3(256), 0, s, probed_dev, nq, nprobe, nlist,
                       pilot, b.hist, b.list_begin, b.job_q, b.job_list, b.job_slot);
    hipLaunchKernelGGL(job_tiles_kernel, dim3((unsigned)((nkeys + 255) / 256)), dim3(256), 0, s, b.list_begin,
                       b.tile_begin, nlist, tq, (TileRec *)b.tiles);
    PSC_HIP_TRY(hipGetLastError());
    return PSC_OK;
}

}  // namespace psc
