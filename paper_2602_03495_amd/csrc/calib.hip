// Calibration of the residual vector of the workload predictor (Section "Residual-Based Prefetching", the
// res_vec equation): res_vec = mean over calibration tokens of h_next - h_cur, as a device reduction.
//
// The sum over tokens is kept in float64 across any number of batches (bf16 differences are exact in fp64 and
// the running sum of up to 2^31 of them loses nothing that survives the final rounding to fp32).  One batch is
// reduced in two fixed-order steps: a grid of (column groups x row slices) writes per-slice partial sums, then
// one thread per column adds the slices in slice order onto the accumulator.  No atomics: the result does not
// depend on scheduling.  HBM-bound: 4 bytes read per (token, column).
#include "moe_common.h"

#define CAL_THREADS 256
#define CAL_COLS 512            // columns per block: 64 lanes x 8 bf16 (one 16-byte load per lane and row)
#define CAL_MAX_SLICES 64

// partial[slice][j] = sum over the rows of the slice of (h_next[r,j] - h_cur[r,j])
__global__ __launch_bounds__(CAL_THREADS) void res_vec_partial_kernel(int n, int d, int rows_per_slice,
                                                                      const uint16_t *__restrict__ h_cur,
                                                                      const uint16_t *__restrict__ h_next,
                                                                      double *__restrict__ partial)
{
    __shared__ double red[CAL_THREADS / 64][CAL_COLS];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j0 = blockIdx.x * CAL_COLS + lane * 8;
    const int r0 = blockIdx.y * rows_per_slice;
    int r1 = r0 + rows_per_slice;
    r1 = r1 > n ? n : r1;
    double acc[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[c] = 0.0;
    if (j0 < d) {
        for (int r = r0 + wave; r < r1; r += CAL_THREADS / 64) {
            const u32x4 a = *reinterpret_cast<const u32x4 *>(h_cur + (size_t)r * d + j0);
            const u32x4 b = *reinterpret_cast<const u32x4 *>(h_next + (size_t)r * d + j0);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                acc[2 * c] += (double)bf16_lo(b[c]) - (double)bf16_lo(a[c]);
                acc[2 * c + 1] += (double)bf16_hi(b[c]) - (double)bf16_hi(a[c]);
            }
        }
    }
#pragma unroll
    for (int c = 0; c < 8; ++c) red[wave][lane * 8 + c] = acc[c];
    __syncthreads();
    for (int c = threadIdx.x; c < CAL_COLS; c += CAL_THREADS) {
        const int j = blockIdx.x * CAL_COLS + c;
        if (j < d) {
            double sum = red[0][c];
#pragma unroll
            for (int w = 1; w < CAL_THREADS / 64; ++w) sum += red[w][c];
            partial[(size_t)blockIdx.y * d + j] = sum;
        }
    }
}

__global__ __launch_bounds__(CAL_THREADS) void res_vec_fold_kernel(int d, int slices, const double *__restrict__ partial,
                                                                   double *__restrict__ acc_sum)
{
    const int j = blockIdx.x * CAL_THREADS + threadIdx.x;
    if (j >= d) return;
    double sum = acc_sum[j];
    for (int s = 0; s < slices; ++s) sum += partial[(size_t)s * d + j];
    acc_sum[j] = sum;
}

__global__ __launch_bounds__(CAL_THREADS) void res_vec_finish_kernel(int d, double n_total, const double *__restrict__ acc_sum,
                                                                     float *__restrict__ res_vec)
{
    const int j = blockIdx.x * CAL_THREADS + threadIdx.x;
    if (j < d) res_vec[j] = (float)(acc_sum[j] / n_total);
}

size_t moe_res_vec_ws_bytes(int d) { return (size_t)CAL_MAX_SLICES * (size_t)d * sizeof(double); }

int moe_res_vec_accumulate_impl(int n, int d, const void *h_cur, const void *h_next, double *acc_sum, void *workspace,
                                hipStream_t st)
{
    if (n == 0) return MOE_OK;
    // slices of at least 64 rows, at most CAL_MAX_SLICES of them
    int slices = (n + 63) / 64;
    slices = slices > CAL_MAX_SLICES ? CAL_MAX_SLICES : slices;
    const int rows_per_slice = (n + slices - 1) / slices;
    slices = (n + rows_per_slice - 1) / rows_per_slice;
    double *partial = (double *)workspace;
    hipLaunchKernelGGL(res_vec_partial_kernel, dim3((d + CAL_COLS - 1) / CAL_COLS, slices), dim3(CAL_THREADS), 0, st, n, d,
                       rows_per_slice, (const uint16_t *)h_cur, (const uint16_t *)h_next, partial);
    MOE_CHECK_LAUNCH();
    hipLaunchKernelGGL(res_vec_fold_kernel, dim3((d + CAL_THREADS - 1) / CAL_THREADS), dim3(CAL_THREADS), 0, st, d, slices,
                       partial, acc_sum);
    MOE_CHECK_LAUNCH();
    return MOE_OK;
}

int moe_res_vec_finish_impl(int d, const double *acc_sum, long long n_total, float *res_vec, hipStream_t st)
{
    hipLaunchKernelGGL(res_vec_finish_kernel, dim3((d + CAL_THREADS - 1) / CAL_THREADS), dim3(CAL_THREADS), 0, st, d,
                       (double)n_total, acc_sum, res_vec);
    MOE_CHECK_LAUNCH();
    return MOE_OK;
}
