// ADC look-up tables and PQ encoding (Section 3 opening; Section 4.2 "ADC").
//
//   lut[r][j][c] = || v_r,j - C[j][c] ||^2        (float32, coordinates in ascending order,
//                                                   one fused multiply-add per coordinate)
//   code[r][j]   = argmin_c of the same quantity   (lowest c on ties)
//
// Both kernels evaluate the distance with the same sequence of float32 operations, so the code
// produced by the encode kernel for a query is exactly the arg-min of that query's table rows.
//
// v_r is row r of the input, optionally re-indexed and with a coarse centroid subtracted
// (residual tables / residual codes of the inverted-file variant, Section 4.3).
#include "common.h"

namespace psc {
namespace {

__device__ __forceinline__ float sub_term(const RowMap &map, int64_t r, int dim, int col)
{
    return map.sub ? map.sub[(int64_t)map.sub_idx[r] * dim + col] : 0.0f;
}

// One workgroup = one sub-quantizer j and ROWS consecutive rows; thread c owns centroid c,
// held in registers (DSUB known at compile time) so the inner loop is pure VALU.
// Table writes are coalesced over c.
template <int DSUB, int ROWS>
__global__ void __launch_bounds__(256)
lut_kernel(const float *__restrict__ cb, int dim, int m, const float *__restrict__ x, int64_t nrows,
           RowMap map, float *__restrict__ lut)
{
    const int j = blockIdx.y;
    const int c = threadIdx.x;
    float cen[DSUB];
    const float *crow = cb + ((int64_t)j * kCentroids + c) * DSUB;
#pragma unroll
    for (int t = 0; t < DSUB; ++t) cen[t] = crow[t];

    __shared__ float vq[ROWS][DSUB];
    const int64_t r0 = (int64_t)blockIdx.x * ROWS;
    for (int e = threadIdx.x; e < ROWS * DSUB; e += 256) {
        const int rr = e / DSUB, t = e % DSUB;
        const int64_t r = r0 + rr;
        float v = 0.f;
        if (r < nrows) {
            const int64_t src = map.row_idx ? (int64_t)map.row_idx[r] : r;
            v = x[src * dim + j * DSUB + t] - sub_term(map, r, dim, j * DSUB + t);
        }
        vq[rr][t] = v;
    }
    __syncthreads();
#pragma unroll 1
    for (int rr = 0; rr < ROWS; ++rr) {
        const int64_t r = r0 + rr;
        if (r >= nrows) break;
        float acc = 0.f;
#pragma unroll
        for (int t = 0; t < DSUB; ++t) {
            const float df = vq[rr][t] - cen[t];
            acc = fmaf(df, df, acc);
        }
        lut[(r * m + j) * kCentroids + c] = acc;
    }
}

// One thread = one row and one sub-quantizer; the sub-codebook sits in LDS and is read by all
// lanes at the same address (broadcast), the row's sub-vector sits in registers.
template <int DSUB>
__global__ void __launch_bounds__(256)
encode_kernel(const float *__restrict__ cb, int dim, int m, const float *__restrict__ x,
              int64_t nrows, RowMap map, uint8_t *__restrict__ codes)
{
    __shared__ float cen[kCentroids * DSUB];
    const int j = blockIdx.y;
    for (int e = threadIdx.x; e < kCentroids * DSUB; e += 256)
        cen[e] = cb[(int64_t)j * kCentroids * DSUB + e];
    __syncthreads();
    const int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (r >= nrows) return;
    float v[DSUB];
    const int64_t src = map.row_idx ? (int64_t)map.row_idx[r] : r;
#pragma unroll
    for (int t = 0; t < DSUB; ++t)
        v[t] = x[src * dim + j * DSUB + t] - sub_term(map, r, dim, j * DSUB + t);
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
    codes[r * m + j] = (uint8_t)bi;
}

template <int DSUB>
int run_lut(const float *cb, int dim, int m, const float *x, int64_t nrows, const RowMap &map,
            float *lut, hipStream_t s)
{
    constexpr int ROWS = 16;
    dim3 grid((unsigned)((nrows + ROWS - 1) / ROWS), (unsigned)m);
    hipLaunchKernelGGL((lut_kernel<DSUB, ROWS>), grid, dim3(256), 0, s, cb, dim, m, x, nrows, map, lut);
    PSC_HIP_TRY(hipGetLastError());
    return PSC_OK;
}

template <int DSUB>
int run_encode(const float *cb, int dim, int m, const float *x, int64_t nrows, const RowMap &map,
               uint8_t *codes, hipStream_t s)
{
    dim3 grid((unsigned)((nrows + 255) / 256), (unsigned)m);
    hipLaunchKernelGGL((encode_kernel<DSUB>), grid, dim3(256), 0, s, cb, dim, m, x, nrows, map, codes);
    PSC_HIP_TRY(hipGetLastError());
    return PSC_OK;
}

}  // namespace

#define PSC_DSUB_SWITCH(dsub, CALL)                                                      \
    switch (dsub) {                                                                      \
    case 1: return CALL(1);                                                              \
    case 2: return CALL(2);                                                              \
    case 4: return CALL(4);                                                              \
    case 6: return CALL(6);                                                              \
    case 8: return CALL(8);                                                              \
    case 12: return CALL(12);                                                            \
    case 16: return CALL(16);                                                            \
    case 24: return CALL(24);                                                            \
    case 32: return CALL(32);                                                            \
    case 48: return CALL(48);                                                            \
    case 64: return CALL(64);                                                            \
    default:                                                                             \
        set_error("unsupported sub-vector length %d (supported: 1,2,4,6,8,12,16,24,32,48,64)", dsub); \
        return PSC_EINVAL;                                                               \
    }

int launch_lut(const float *cb_dev, int dim, int m, const float *x_dev, int64_t nrows,
               const RowMap &map, float *lut_dev, hipStream_t s)
{
    if (nrows == 0) return PSC_OK;
    if ((nrows + 15) / 16 > 0x7fffffffLL) {
        set_error("too many rows for one table launch");
        return PSC_EINVAL;
    }
#define CALL(DS) run_lut<DS>(cb_dev, dim, m, x_dev, nrows, map, lut_dev, s)
    PSC_DSUB_SWITCH(dim / m, CALL)
#undef CALL
}

int launch_encode(const float *cb_dev, int dim, int m, const float *x_dev, int64_t nrows,
                  const RowMap &map, uint8_t *codes_dev, hipStream_t s)
{
    if (nrows == 0) return PSC_OK;
    if ((nrows + 255) / 256 > 0x7fffffffLL) {
        set_error("too many rows for one encode launch");
        return PSC_EINVAL;
    }
#define CALL(DS) run_encode<DS>(cb_dev, dim, m, x_dev, nrows, map, codes_dev, s)
    PSC_DSUB_SWITCH(dim / m, CALL)
#undef CALL
}

}  // namespace psc
