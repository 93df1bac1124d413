// Lloyd k-means on the GPU for the product quantizer (Section 3, opening: one k-means of 256
// centroids per sub-space) and for the coarse quantizer of the inverted file (Section 4.3).
// Offline work, left of the scan: the search path never comes here.
//
// One iteration = assignment (nearest centroid in float32, lowest number on ties) + the sums and
// counts of every cell; the new centroid is sum / count in double precision, rounded to float32.
// Sums are order-dependent in their last bits (atomic adds), so two runs agree to rounding, not
// bit for bit.
#include <hip/hip_runtime.h>

#include "common.h"

namespace psc {

namespace {

// ---------------------------------------------------------------------------------------------
// Product quantizer: grid (row blocks, m).  A workgroup keeps sub-codebook j and a private copy of
// its cells' sums (float32: a workgroup adds a few members per cell) and counts in LDS, walks its
// share of the rows (one row per thread and turn), and adds its sums to the global ones (double)
// at the end.  Per row it also stores the cell and the distance, for the refill of empty cells.
// ---------------------------------------------------------------------------------------------
template <int DSUB>
__global__ void __launch_bounds__(256)
pq_lloyd_step_kernel(const float *__restrict__ cb, int dim, int m, const float *__restrict__ x, int64_t n,
                     uint8_t *__restrict__ cell, float *__restrict__ dmin, double *__restrict__ gsum,
                     uint32_t *__restrict__ gcount, double *__restrict__ gobj)
{
    extern __shared__ float smem[];
    float *cen = smem;                                     // [256][DSUB]
    float *sum = smem + kCentroids * DSUB;                 // [256][DSUB]
    uint32_t *cnt = (uint32_t *)(smem + 2 * kCentroids * DSUB);  // [256]
    const int j = blockIdx.y, tid = threadIdx.x;
    for (int e = tid; e < kCentroids * DSUB; e += 256) {
        cen[e] = cb[(int64_t)j * kCentroids * DSUB + e];
        sum[e] = 0.f;
    }
    cnt[tid] = 0u;
    __syncthreads();
    double obj = 0.0;
    for (int64_t r = (int64_t)blockIdx.x * 256 + tid; r < n; r += (int64_t)gridDim.x * 256) {
        float v[DSUB];
#pragma unroll
        for (int t = 0; t < DSUB; ++t) v[t] = x[r * dim + j * DSUB + t];
        float best = __builtin_inff();
        int bi = 0;
#pragma unroll 2
        for (int c = 0; c < kCentroids; ++c) {
            float acc = 0.f;
#pragma unroll
            for (int t = 0; t < DSUB; ++t) {
                const float df = v[t] - cen[c * DSUB + t];
                acc = fmaf(df, df, acc);
            }
            if (acc < best) {
                best = acc;
                bi = c;
            }
        }
        cell[r * m + j] = (uint8_t)bi;
        dmin[r * m + j] = best;
        obj += (double)best;
#pragma unroll
        for (int t = 0; t < DSUB; ++t) unsafeAtomicAdd(&sum[bi * DSUB + t], v[t]);
        atomicAdd(&cnt[bi], 1u);
    }
    __syncthreads();
    for (int e = tid; e < kCentroids * DSUB; e += 256)
        if (cnt[e / DSUB] != 0u) unsafeAtomicAdd(&gsum[(int64_t)j * kCentroids * DSUB + e], (double)sum[e]);
    if (cnt[tid] != 0u) atomicAdd(&gcount[j * kCentroids + tid], cnt[tid]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) obj += __shfl_xor(obj, off, 64);
    if ((tid & 63) == 0) unsafeAtomicAdd(&gobj[j], obj);
}

// The 256 starting centroids of every sub-quantizer: sub-vector j of row rows[j][c].
__global__ void __launch_bounds__(256)
pq_gather_start_kernel(const float *__restrict__ x, int dim, int dsub, const int64_t *__restrict__ rows,
                       float *__restrict__ cb)
{
    const int j = blockIdx.x, c = threadIdx.x;
    const float *src = x + rows[j * kCentroids + c] * dim + j * dsub;
    float *dst = cb + ((int64_t)j * kCentroids + c) * dsub;
    for (int t = 0; t < dsub; ++t) dst[t] = src[t];
}

// Refill of an empty cell, step 1: the member of cell `big` of sub-quantizer j that lies farthest
// from its centroid, lowest row on equal distance.  key = (distance bits << 32) | ~row, maximised.
__global__ void __launch_bounds__(256)
pq_farthest_member_kernel(const uint8_t *__restrict__ cell, const float *__restrict__ dmin, int64_t n, int m,
                          int j, int big, unsigned long long *__restrict__ key)
{
    unsigned long long best = 0ull;
    for (int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x; r < n; r += (int64_t)gridDim.x * 256)
        if (cell[r * m + j] == (uint8_t)big) {
            const unsigned long long k =
                ((unsigned long long)__float_as_uint(dmin[r * m + j]) << 32) | (0xffffffffu - (uint32_t)r);
            best = k > best ? k : best;
        }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const unsigned long long o = __shfl_xor(best, off, 64);
        best = o > best ? o : best;
    }
    if ((threadIdx.x & 63) == 0 && best != 0ull) atomicMax(key, best);
}

// Step 2: row `far` becomes the only member of the empty cell c (the sum and count of the cell
// it leaves stay as they are: that cell's mean still includes it in this iteration).
__global__ void pq_move_member_kernel(const float *__restrict__ x, int dim, int dsub, int m, int j, int64_t far,
                                      int c, uint8_t *__restrict__ cell, float *__restrict__ dmin,
                                      double *__restrict__ gsum, uint32_t *__restrict__ gcount)
{
    const int t = threadIdx.x;
    if (t < dsub) gsum[((int64_t)j * kCentroids + c) * dsub + t] = (double)x[far * dim + j * dsub + t];
    if (t == 0) {
        cell[far * m + j] = (uint8_t)c;
        dmin[far * m + j] = 0.f;
        gcount[j * kCentroids + c] = 1u;
    }
}

// cent[c] = sum[c] / count[c] for the cells that have members; the others keep their centroid.
__global__ void __launch_bounds__(256)
centroid_update_kernel(const double *__restrict__ gsum, const uint32_t *__restrict__ gcount, int64_t ncell,
                       int d, float *__restrict__ cent)
{
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= ncell * d) return;
    const uint32_t cnt = gcount[e / d];
    if (cnt != 0u) cent[e] = (float)(gsum[e] / (double)cnt);
}

// ---------------------------------------------------------------------------------------------
// Coarse quantizer: the assignment comes from the nearest-centroid kernel; this adds every row to
// its cell.  One thread per (row, 4 coordinates), atomics straight to the global sums: the cells
// are too many for private copies, and a row's coordinates go to consecutive addresses.
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
coarse_accumulate_kernel(const float *__restrict__ x, int64_t n, int dim, const int32_t *__restrict__ assign,
                         double *__restrict__ gsum, uint32_t *__restrict__ gcount)
{
    const int q4 = dim / 4;
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= n * q4) return;
    const int64_t r = e / q4;
    const int t4 = (int)(e - r * q4);
    const int c = assign[r];
    const float4 v = *(const float4 *)(x + r * dim + 4 * t4);
    double *s = gsum + (int64_t)c * dim + 4 * t4;
    unsafeAtomicAdd(s + 0, (double)v.x);
    unsafeAtomicAdd(s + 1, (double)v.y);
    unsafeAtomicAdd(s + 2, (double)v.z);
    unsafeAtomicAdd(s + 3, (double)v.w);
    if (t4 == 0) atomicAdd(&gcount[c], 1u);
}

__global__ void __launch_bounds__(256)
gather_rows_kernel(const float *__restrict__ x, int dim, const int64_t *__restrict__ rows, int64_t nrows,
                   float *__restrict__ out)
{
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= nrows * dim) return;
    const int64_t c = e / dim;
    out[e] = x[rows[c] * dim + (e - c * dim)];
}

// Refill of an empty coarse cell: the lowest-numbered member of cell `big`.
__global__ void __launch_bounds__(256)
coarse_first_member_kernel(const int32_t *__restrict__ assign, int64_t n, int big, unsigned long long *__restrict__ key)
{
    unsigned long long best = 0ull;
    for (int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x; r < n; r += (int64_t)gridDim.x * 256)
        if (assign[r] == big) {
            const unsigned long long k = (1ull << 32) | (0xffffffffu - (uint32_t)r);
            best = k > best ? k : best;
        }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const unsigned long long o = __shfl_xor(best, off, 64);
        best = o > best ? o : best;
    }
    if ((threadIdx.x & 63) == 0 && best != 0ull) atomicMax(key, best);
}

__global__ void coarse_move_member_kernel(const float *__restrict__ x, int dim, int64_t far, int c,
                                          int32_t *__restrict__ assign, double *__restrict__ gsum,
                                          uint32_t *__restrict__ gcount)
{
    for (int t = threadIdx.x; t < dim; t += blockDim.x) gsum[(int64_t)c * dim + t] = (double)x[far * dim + t];
    if (threadIdx.x == 0) {
        assign[far] = c;
        gcount[c] = 1u;
    }
}

// The mean of the centroids, appended as row ncent: the reference point of the matrix-core
// distance kernel.  One workgroup per coordinate, a fixed order of additions.
__global__ void __launch_bounds__(256)
mean_centroid_kernel(float *__restrict__ cent, int ncent, int dim)
{
    __shared__ double part[4];
    const int t = blockIdx.x;
    double acc = 0.0;
    for (int c = threadIdx.x; c < ncent; c += 256) acc += (double)cent[(int64_t)c * dim + t];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) cent[(int64_t)ncent * dim + t] = (float)((part[0] + part[1] + part[2] + part[3]) / ncent);
}

template <int DSUB>
int run_pq_step(const float *cb, int dim, int m, const float *x, int64_t n, uint8_t *cell, float *dmin,
                double *gsum, uint32_t *gcount, double *gobj, hipStream_t s)
{
    const size_t lds = (size_t)(2 * kCentroids * DSUB + kCentroids) * sizeof(float);
    if (lds > 48 * 1024)
        PSC_HIP_TRY(hipFuncSetAttribute((const void *)pq_lloyd_step_kernel<DSUB>,
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    const int64_t want = (n + 255) / 256, cap = 2048 / m;
    dim3 grid((unsigned)(want < cap ? want : cap), (unsigned)m);
    hipLaunchKernelGGL((pq_lloyd_step_kernel<DSUB>), grid, dim3(256), lds, s, cb, dim, m, x, n, cell, dmin, gsum,
                       gcount, gobj);
    PSC_HIP_TRY(hipGetLastError());
    return PSC_OK;
}

}  // namespace

int launch_pq_lloyd_step(const float *cb_dev, int dim, int m, const float *x_dev, int64_t n, uint8_t *cell_dev,
                         float *dmin_dev, double *sum_dev, uint32_t *count_dev, double *obj_dev, hipStream_t s)
{
    const size_t ncell = (size_t)m * kCentroids;
    PSC_HIP_TRY(hipMemsetAsync(sum_dev, 0, ncell * (size_t)(dim / m) * sizeof(double), s));
    PSC_HIP_TRY(hipMemsetAsync(count_dev, 0, ncell * sizeof(uint32_t), s));
    PSC_HIP_TRY(hipMemsetAsync(obj_dev, 0, (size_t)m * sizeof(double), s));
#define CALL(DS) run_pq_step<DS>(cb_dev, dim, m, x_dev, n, cell_dev, dmin_dev, sum_dev, count_dev, obj_dev, s)
    switch (dim / m) {
    case 1: return CALL(1);
    case 2: return CALL(2);
    case 4: return CALL(4);
    case 6: return CALL(6);
    case 8: return CALL(8);
    case 12: return CALL(12);
    case 16: return CALL(16);
    case 24: return CALL(24);
    case 32: return CALL(32);
    case 48: return CALL(48);
    case 64: return CALL(64);
    default:
        set_error("unsupported sub-vector length %d (supported: 1,2,4,6,8,12,16,24,32,48,64)", dim / m);
        return PSC_EINVAL;
    }
#undef CALL
}

int launch_pq_gather_start(const float *x_dev, int dim, int m, const int64_t *rows_dev, float *cb_dev, hipStream_t s)
{
    hipLaunchKernelGGL(pq_gather_start_kernel, dim3((unsigned)m), dim3(kCentroids), 0, s, x_dev, dim, dim / m,
                       rows_dev, cb_dev);
    PSC_HIP_TRY(hipGetLastError());
    return PSC_OK;
}

int launch_pq_refill(const float *x_dev, int64_t n, int dim, int m, int j, int big, int c, uint8_t *cell_dev,
                     float *dmin_dev, double *sum_dev, uint32_t *count_dev, unsigned long long *key_dev,
                     hipStream_t s)
{
    PSC_HIP_TRY(hipMemsetAsync(key_dev, 0, sizeof(unsigned long long), s));
    const int64_t want = (n + 255) / 256;
    hipLaunchKernelGGL(pq_farthest_member_kernel, dim3((unsigned)(want < 1024 ? want : 1024)), dim3(256), 0, s,
                       cell_dev, dmin_dev, n, m, j, big, key_dev);
    PSC_HIP_TRY(hipGetLastError());
    unsigned long long key = 0;
    PSC_HIP_TRY(hipMemcpyAsync(&key, key_dev, sizeof key, hipMemcpyDeviceToHost, s));
    PSC_HIP_TRY(hipStreamSynchronize(s));
    if (key == 0ull) return PSC_OK;  // the cell has no member: nothing to move
    const int64_t far = (int64_t)(0xffffffffu - (uint32_t)(key & 0xffffffffull));
    hipLaunchKernelGGL(pq_move_member_kernel, dim3(1), dim3(64), 0, s, x_dev, dim, dim / m, m, j, far, c,
                       cell_dev, dmin_dev, sum_dev, count_dev);
    PSC_HIP_TRY(hipGetLastError());
    return PSC_OK;
}

int launch_centroid_update(const double *sum_dev, const uint32_t *count_dev, int64_t ncell, int d, float *cent_dev,
                           hipStream_t s)
{
    const int64_t total = ncell * d;
    hipLaunchKernelGGL(centroid_update_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, sum_dev,
                       count_dev, ncell, d, cent_dev);
    PSC_HIP_TRY(hipGetLastError());
    return PSC_OK;
}

int launch_gather_rows(const float *x_dev, int dim, const int64_t *rows_dev, int64_t nrows, float *out_dev,
                       hipStream_t s)
{
    const int64_t total = nrows * dim;
    hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, x_dev, dim,
                       rows_dev, nrows, out_dev);
    PSC_HIP_TRY(hipGetLastError());
    return PSC_OK;
}

int launch_coarse_accumulate(const float *x_dev, int64_t n, int dim, const int32_t *assign_dev, int ncent,
                             double *sum_dev, uint32_t *count_dev, hipStream_t s)
{
    PSC_HIP_TRY(hipMemsetAsync(sum_dev, 0, (size_t)ncent * dim * sizeof(double), s));
    PSC_HIP_TRY(hipMemsetAsync(count_dev, 0, (size_t)ncent * sizeof(uint32_t), s));
    const int64_t total = n * (dim / 4), blocks = (total + 255) / 256;
    if (blocks > 0x7fffffffLL) {
        set_error("too many training rows for one launch");
        return PSC_EINVAL;
    }
    hipLaunchKernelGGL(coarse_accumulate_kernel, dim3((unsigned)blocks), dim3(256), 0, s, x_dev, n, dim, assign_dev,
                       sum_dev, count_dev);
    PSC_HIP_TRY(hipGetLastError());
    return PSC_OK;
}

int launch_coarse_refill(const float *x_dev, int64_t n, int dim, int big, int c, int32_t *assign_dev,
                         double *sum_dev, uint32_t *count_dev, unsigned long long *key_dev, hipStream_t s)
{
    PSC_HIP_TRY(hipMemsetAsync(key_dev, 0, sizeof(unsigned long long), s));
    const int64_t want = (n + 255) / 256;
    hipLaunchKernelGGL(coarse_first_member_kernel, dim3((unsigned)(want < 1024 ? want : 1024)), dim3(256), 0, s,
                       assign_dev, n, big, key_dev);
    PSC_HIP_TRY(hipGetLastError());
    unsigned long long key = 0;
    PSC_HIP_TRY(hipMemcpyAsync(&key, key_dev, sizeof key, hipMemcpyDeviceToHost, s));
    PSC_HIP_TRY(hipStreamSynchronize(s));
    if (key == 0ull) return PSC_OK;
    const int64_t far = (int64_t)(0xffffffffu - (uint32_t)(key & 0xffffffffull));
    hipLaunchKernelGGL(coarse_move_member_kernel, dim3(1), dim3(256), 0, s, x_dev, dim, far, c, assign_dev,
                       sum_dev, count_dev);
    PSC_HIP_TRY(hipGetLastError());
    return PSC_OK;
}

int launch_mean_centroid(float *cent_dev, int ncent, int dim, hipStream_t s)
{
    hipLaunchKernelGGL(mean_centroid_kernel, dim3((unsigned)dim), dim3(256), 0, s, cent_dev, ncent, dim);
    PSC_HIP_TRY(hipGetLastError());
    return PSC_OK;
}

}  // namespace psc
