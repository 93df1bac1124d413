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
    if (map.k2 > 0) {  // multi-index cell a * k2 + b: the cell centroid is (sub[a], sub_b[b]), dim / 2 floats each
        const int cell = map.sub_idx[r], half = dim / 2;
        const int a = cell / map.k2, b = cell - a * map.k2;
        return col < half ? map.sub[(int64_t)a * half + col] : map.sub_b[(int64_t)b * half + col - half];
    }
    return map.sub ? map.sub[(int64_t)(map.sub_idx ? map.sub_idx[r] : 0) * dim + col] : 0.0f;
}

// One workgroup = one sub-quantizer j and ROWS consecutive rows; thread c owns centroid c,
// held in registers (DSUB known at compile time) so the inner loop is pure VALU.
// Table writes are coalesced over c.
// CROSS: instead of the squared distance, the part of it that depends on the centroid,
//   || c ||^2 - 2 v . c  =  sum_t c_t (c_t - 2 v_t),
// which the inverted-file scan completes with a per-list table and a number per (query, list).
template <int DSUB, int ROWS, bool CROSS>
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
            if constexpr (CROSS) {
                acc = fmaf(cen[t], cen[t] - 2.0f * vq[rr][t], acc);
            } else {
                const float df = vq[rr][t] - cen[t];
                acc = fmaf(df, df, acc);
            }
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

// ---------------------------------------------------------------------------------------------
// Table construction as a dense contraction on the matrix cores (full float32 MFMA):
//     || q - c ||^2 = || q' ||^2 - 2 q'.c' + || c' ||^2,     q' = q - mu_j,  c' = c - mu_j
// where mu_j is the mean centroid of sub-quantizer j (distances do not change under a common
// shift; centring keeps the three terms small, which keeps the cancellation error small).
// One workgroup = 32 rows x the 256 centroids of one sub-quantizer; each of its 4 waves owns two
// 32 x 32 output tiles and runs DSUB/2 v_mfma_f32_32x32x2f32 steps per tile.
//
// v_mfma_f32_32x32x2f32 operand layout (wave64, lane l): A[i][k] with i = l % 32, k = l / 32;
// B[k][j] with k = l / 32, j = l % 32; D[i][j] in 16 registers, register v holding row
// i = 8 * (v / 4) + 4 * (l / 32) + v % 4, column j = l % 32.
// ---------------------------------------------------------------------------------------------
typedef float f32x16 __attribute__((ext_vector_type(16)));
// Entries below this share of || q' ||^2 + || c' ||^2 are recomputed by direct differences; the
// others keep a relative error of a few float32 roundings x 16 (about 3e-6 at worst).
constexpr float kRefineBelow = 1.0f / 16.0f;

template <int DSUB>
__global__ void __launch_bounds__(256)
lut_mfma_kernel(const float *__restrict__ cb, const float *__restrict__ cbc /* centred codebook */,
                const float *__restrict__ mu, int dim, int m, const float *__restrict__ x, int64_t nrows,
                float *__restrict__ lut)
{
    static_assert(DSUB % 2 == 0, "two coordinates per MFMA step");
    constexpr int KS = DSUB / 2;
    __shared__ float qn_s[4][32];
    const int j = blockIdx.y;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int half = lane >> 5, col = lane & 31;
    const int64_t r0 = (int64_t)blockIdx.x * 32;

    // A operand: row r0 + col, coordinates half, 2 + half, 4 + half, ... (centred)
    float a[KS];
    {
        const int64_t r = r0 + col;
        const float *xr = x + (r < nrows ? r : nrows - 1) * dim + j * DSUB;
        const float *mj = mu + j * DSUB;
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) a[kk] = xr[2 * kk + half] - mj[2 * kk + half];
    }
    // || q' ||^2 of row `col`: this lane's half of the coordinates plus the other half's
    float qn = 0.f;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) qn = fmaf(a[kk], a[kk], qn);
    qn += __shfl_xor(qn, 32, 64);
    if (half == 0) qn_s[wave][col] = qn;
    __builtin_amdgcn_wave_barrier();

#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const int c0 = (wave * 2 + t) * 32;
        const float *cr = cbc + ((int64_t)j * kCentroids + c0 + col) * DSUB;
        float b[KS];
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) b[kk] = cr[2 * kk + half];
        float cn = 0.f;
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) cn = fmaf(b[kk], b[kk], cn);
        cn += __shfl_xor(cn, 32, 64);
        f32x16 acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[kk], b[kk], acc, 0, 0, 0);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int i = 8 * (v / 4) + 4 * half + v % 4;
            const int64_t r = r0 + i;
            if (r < nrows) {
                const float sum = qn_s[wave][i] + cn;
                float d = fmaf(-2.0f, acc[v], sum);
                if (d < kRefineBelow * sum) {
                    // the three terms have cancelled to less than a sixteenth of their size: what
                    // is left has lost four bits or more, so this entry (a centroid close to the
                    // query -- the entries that decide the query's code and its nearest
                    // neighbours) is taken by direct differences instead, in the operation order
                    // of the encoding kernel
                    const float *xr = x + r * dim + j * DSUB;
                    const float *cr2 = cb + ((int64_t)j * kCentroids + c0 + col) * DSUB;
                    float e = 0.f;
#pragma unroll
                    for (int t = 0; t < DSUB; ++t) {
                        const float df = xr[t] - cr2[t];
                        e = fmaf(df, df, e);
                    }
                    d = e;
                }
                lut[(r * m + j) * kCentroids + c0 + col] = d > 0.f ? d : 0.f;
            }
        }
    }
}

// code[r][j] = index of the smallest entry of table row (r, j), lowest index on ties: the query's
// own code, taken from the very table the scan will use.  One wave per row.
__global__ void __launch_bounds__(256)
row_argmin_kernel(const float *__restrict__ lut, int64_t nrows_total, uint8_t *__restrict__ codes)
{
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= nrows_total) return;
    const int lane = threadIdx.x & 63;
    const float4 v = *(const float4 *)(lut + row * kCentroids + lane * 4);
    float best = v.x;
    int bi = lane * 4;
    if (v.y < best) { best = v.y; bi = lane * 4 + 1; }
    if (v.z < best) { best = v.z; bi = lane * 4 + 2; }
    if (v.w < best) { best = v.w; bi = lane * 4 + 3; }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float ob = __shfl_xor(best, off, 64);
        const int oi = __shfl_xor(bi, off, 64);
        if (ob < best || (ob == best && oi < bi)) {
            best = ob;
            bi = oi;
        }
    }
    if (lane == 0) codes[row] = (uint8_t)bi;
}

template <int DSUB>
int run_lut_mfma(const float *cb, const float *cbc, const float *mu, int dim, int m, const float *x, int64_t nrows,
                 float *lut, hipStream_t s)
{
    dim3 grid((unsigned)((nrows + 31) / 32), (unsigned)m);
    hipLaunchKernelGGL((lut_mfma_kernel<DSUB>), grid, dim3(256), 0, s, cb, cbc, mu, dim, m, x, nrows, lut);
    PSC_HIP_TRY(hipGetLastError());
    return PSC_OK;
}

template <int DSUB>
int run_lut(const float *cb, int dim, int m, const float *x, int64_t nrows, const RowMap &map, bool cross,
            float *lut, hipStream_t s)
{
    constexpr int ROWS = 16;
    dim3 grid((unsigned)((nrows + ROWS - 1) / ROWS), (unsigned)m);
    if (cross)
        hipLaunchKernelGGL((lut_kernel<DSUB, ROWS, true>), grid, dim3(256), 0, s, cb, dim, m, x, nrows, map, lut);
    else
        hipLaunchKernelGGL((lut_kernel<DSUB, ROWS, false>), grid, dim3(256), 0, s, cb, dim, m, x, nrows, map, lut);
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
               const RowMap &map, bool cross, float *lut_dev, hipStream_t s)
{
    if (nrows == 0) return PSC_OK;
    if ((nrows + 15) / 16 > 0x7fffffffLL) {
        set_error("too many rows for one table launch");
        return PSC_EINVAL;
    }
#define CALL(DS) run_lut<DS>(cb_dev, dim, m, x_dev, nrows, map, cross, lut_dev, s)
    PSC_DSUB_SWITCH(dim / m, CALL)
#undef CALL
}

int launch_lut_mfma(const float *cb_dev, const float *cbc_dev, const float *mu_dev, int dim, int m,
                    const float *x_dev, int64_t nrows, float *lut_dev, hipStream_t s)
{
    if (nrows == 0) return PSC_OK;
    if ((nrows + 31) / 32 > 0x7fffffffLL) {
        set_error("too many rows for one table launch");
        return PSC_EINVAL;
    }
    switch (dim / m) {
    case 2: return run_lut_mfma<2>(cb_dev, cbc_dev, mu_dev, dim, m, x_dev, nrows, lut_dev, s);
    case 4: return run_lut_mfma<4>(cb_dev, cbc_dev, mu_dev, dim, m, x_dev, nrows, lut_dev, s);
    case 6: return run_lut_mfma<6>(cb_dev, cbc_dev, mu_dev, dim, m, x_dev, nrows, lut_dev, s);
    case 8: return run_lut_mfma<8>(cb_dev, cbc_dev, mu_dev, dim, m, x_dev, nrows, lut_dev, s);
    case 12: return run_lut_mfma<12>(cb_dev, cbc_dev, mu_dev, dim, m, x_dev, nrows, lut_dev, s);
    case 16: return run_lut_mfma<16>(cb_dev, cbc_dev, mu_dev, dim, m, x_dev, nrows, lut_dev, s);
    case 24: return run_lut_mfma<24>(cb_dev, cbc_dev, mu_dev, dim, m, x_dev, nrows, lut_dev, s);
    case 32: return run_lut_mfma<32>(cb_dev, cbc_dev, mu_dev, dim, m, x_dev, nrows, lut_dev, s);
    case 48: return run_lut_mfma<48>(cb_dev, cbc_dev, mu_dev, dim, m, x_dev, nrows, lut_dev, s);
    case 64: return run_lut_mfma<64>(cb_dev, cbc_dev, mu_dev, dim, m, x_dev, nrows, lut_dev, s);
    default:
        set_error("the matrix-core table kernel needs an even sub-vector length, got %d", dim / m);
        return PSC_EINVAL;
    }
}

int launch_row_argmin(const float *lut_dev, int64_t nrows_total, uint8_t *codes_dev, hipStream_t s)
{
    if (nrows_total == 0) return PSC_OK;
    if ((nrows_total + 3) / 4 > 0x7fffffffLL) {
        set_error("too many table rows");
        return PSC_EINVAL;
    }
    hipLaunchKernelGGL(row_argmin_kernel, dim3((unsigned)((nrows_total + 3) / 4)), dim3(256), 0, s, lut_dev,
                       nrows_total, codes_dev);
    PSC_HIP_TRY(hipGetLastError());
    return PSC_OK;
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
