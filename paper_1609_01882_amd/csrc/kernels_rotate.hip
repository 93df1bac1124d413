// Linear transformation in front of the product quantizer (Section 4.3: an optimized rotation
// before encoding; the additional results reduce the dimension inside the same transformation,
// e.g. 128-D -> 64-D in front of 8 sub-quantizers):
//
//     y[r][c] = sum_t x[r][t] * R[c][t]          x [n][din], R [dout][din], y [n][dout]
//
// a dense contraction, so it runs on the matrix cores in full float32 (v_mfma_f32_32x32x2f32;
// operand layout: A[i][k] with i = lane % 32, k = lane / 32; B[k][j] with k = lane / 32,
// j = lane % 32; D[i][j] in 16 registers, register v = row 8 * (v / 4) + 4 * (lane / 32) + v % 4,
// column j = lane % 32).  One workgroup = 4 waves x 32 rows and up to 128 output columns (four
// accumulator tiles per wave); the input dimension is walked in chunks of 64 coordinates held in
// registers.  The matrix is stored transposed and zero-padded (rt [din_pad][dout_pad], din_pad a
// multiple of 64, dout_pad of 32), so a B operand is one coalesced 128-byte read per half-wave and
// stays in the caches (the matrix is a few hundred KB at most).
#include "common.h"

namespace psc {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
constexpr int kChunk = 64;      // input coordinates per step (32 MFMA steps of 2)
constexpr int kColTiles = 4;    // 32-column output tiles per workgroup

__global__ void __launch_bounds__(256)
rotate_mfma_kernel(const float *__restrict__ x, int64_t n, int din, const float *__restrict__ rt, int din_pad,
                   int dout, int dout_pad, float *__restrict__ y)
{
    const int tid = (int)threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int half = lane >> 5, col = lane & 31;
    const int64_t r0 = (int64_t)blockIdx.x * 128 + wave * 32;
    const int c_base = (int)blockIdx.y * (32 * kColTiles);
    const int64_t r = r0 + col;
    const float *xr = x + (r < n ? r : n - 1) * (int64_t)din;

    f32x16 acc[kColTiles];
#pragma unroll
    for (int t = 0; t < kColTiles; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;

    for (int kc = 0; kc < din_pad; kc += kChunk) {
        float a[kChunk / 2];
#pragma unroll
        for (int kk = 0; kk < kChunk / 2; ++kk) {
            const int t = kc + 2 * kk + half;
            a[kk] = t < din ? xr[t] : 0.f;
        }
#pragma unroll
        for (int t = 0; t < kColTiles; ++t) {
            const int c0 = c_base + 32 * t;
            if (c0 >= dout_pad) break;  // (uniform over the workgroup)
            const float *b = rt + (int64_t)(kc + half) * dout_pad + c0 + col;
#pragma unroll
            for (int kk = 0; kk < kChunk / 2; ++kk)
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[kk], b[(int64_t)(2 * kk) * dout_pad], acc[t], 0, 0, 0);
        }
    }
#pragma unroll
    for (int t = 0; t < kColTiles; ++t) {
        const int c = c_base + 32 * t + col;
        if (c >= dout) continue;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int64_t row = r0 + 8 * (v / 4) + 4 * half + v % 4;
            if (row < n) y[row * dout + c] = acc[t][v];
        }
    }
}

}  // namespace

int launch_rotate(const float *x_dev, int64_t n, int din, const float *rt_dev, int din_pad, int dout, int dout_pad,
                  float *y_dev, hipStream_t s)
{
    if (n == 0) return PSC_OK;
    PSC_REQUIRE((n + 127) / 128 <= 0x7fffffffLL, "too many rows for one transformation launch");
    PSC_REQUIRE(din_pad % kChunk == 0 && dout_pad % 32 == 0 && din <= din_pad && dout <= dout_pad, "bad matrix padding");
    dim3 grid((unsigned)((n + 127) / 128), (unsigned)((dout_pad + 32 * kColTiles - 1) / (32 * kColTiles)));
    hipLaunchKernelGGL(rotate_mfma_kernel, grid, dim3(256), 0, s, x_dev, n, din, rt_dev, din_pad, dout, dout_pad, y_dev);
    PSC_HIP_TRY(hipGetLastError());
    return PSC_OK;
}

}  // namespace psc
