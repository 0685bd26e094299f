// Variance indicator (LLM-PQ, arXiv 2403.01136, Sec. 4.2, Theorem 1 and Eq. 3): the extra output variance of a
// linear operator under b-bit weight quantisation is estimated as D_W * S_W(b)^2 * G(X), G(X) = Var[X] / 4
// (deterministic rounding) or (E[X]^2 + Var[X]) / 6 (stochastic rounding).
//
// Everything it needs is a few reductions, bound by reading W and X once from HBM:
//   per row of W:  sum over its 128-column groups of (max - min)^2, max |w|, min, max   (one wave per row)
//   over X:        sum x, sum x^2                                                       (fp64 per lane)
// and one small kernel that adds the per-row values in fp64 and evaluates the eight forms: the printed
// one-scale-per-matrix form and the form with the quantiser's own granularity (a scale per (row, 128
// columns) group, or per row for the symmetric scheme), for bits 3, 4, 8 and symmetric 8.
#include <algorithm>
#include "lpq_common.h"
#include "lpq_device.h"

namespace lpq {

namespace {

// row statistics: stats[4 * n + {0,1,2,3}] = sum of group ranges squared, max |w|, min, max
__global__ __launch_bounds__(256) void indicator_row_stats_kernel(const uint16_t* __restrict__ w, int K, int N, float* __restrict__ stats)
{
    const int lane = threadIdx.x & 63;
    const long n = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (n >= N) return;
    const uint16_t* row = w + n * K;
    float range_sq = 0.0f, amax = 0.0f, lo_all = INFINITY, hi_all = -INFINITY;
    for (int k = 8 * lane; k < K; k += 512) {          // 16 lanes cover one 128-column group
        const h8 t = *reinterpret_cast<const h8*>(row + k);
        float lo = (float)t[0], hi = lo;
#pragma unroll
        for (int e = 1; e < 8; ++e) { lo = fminf(lo, (float)t[e]); hi = fmaxf(hi, (float)t[e]); }
#pragma unroll
        for (int off = 1; off < 16; off <<= 1) { lo = fminf(lo, __shfl_xor(lo, off)); hi = fmaxf(hi, __shfl_xor(hi, off)); }
        if ((lane & 15) == 0) range_sq += (hi - lo) * (hi - lo);
        lo_all = fminf(lo_all, lo);
        hi_all = fmaxf(hi_all, hi);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        range_sq += __shfl_xor(range_sq, off);
        lo_all = fminf(lo_all, __shfl_xor(lo_all, off));
        hi_all = fmaxf(hi_all, __shfl_xor(hi_all, off));
    }
    amax = fmaxf(fabsf(lo_all), fabsf(hi_all));
    if (lane == 0) {
        float* s = stats + 4 * n;
        s[0] = range_sq; s[1] = amax; s[2] = lo_all; s[3] = hi_all;
    }
}

// partial sums of x and x^2 per workgroup, in fp64
__global__ __launch_bounds__(256) void indicator_x_sums_kernel(const uint16_t* __restrict__ x, long n8, double* __restrict__ part)
{
    __shared__ double red[2][4];
    double s = 0.0, q = 0.0;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n8; i += (long)gridDim.x * 256) {
        const h8 t = *reinterpret_cast<const h8*>(x + 8 * i);
#pragma unroll
        for (int e = 0; e < 8; ++e) { const double v = (double)(float)t[e]; s += v; q += v * v; }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) { s += __shfl_xor(s, off); q += __shfl_xor(q, off); }
    if ((threadIdx.x & 63) == 0) { red[0][threadIdx.x >> 6] = s; red[1][threadIdx.x >> 6] = q; }
    __syncthreads();
    if (threadIdx.x == 0) {
        part[2 * blockIdx.x] = (red[0][0] + red[0][1]) + (red[0][2] + red[0][3]);
        part[2 * blockIdx.x + 1] = (red[1][0] + red[1][1]) + (red[1][2] + red[1][3]);
    }
}

__device__ __forceinline__ double block_sum_f64(double v, double* red)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return (red[0] + red[1]) + (red[2] + red[3]);
}

// one workgroup: add the rows' statistics and the partial sums of X in fp64, evaluate the eight forms
__global__ __launch_bounds__(256) void indicator_finish_kernel(const float* __restrict__ stats, int K, int N, const double* __restrict__ xpart,
                                                               int x_blocks, double x_count, int stochastic, double* __restrict__ omega)
{
    __shared__ double red[4];
    __shared__ float redf[2][4];
    double range_sq = 0.0, amax_sq = 0.0;
    float lo = INFINITY, hi = -INFINITY;
    for (int n = threadIdx.x; n < N; n += 256) {
        const float* s = stats + 4 * (long)n;
        range_sq += (double)s[0];
        amax_sq += (double)s[1] * (double)s[1];
        lo = fminf(lo, s[2]);
        hi = fmaxf(hi, s[3]);
    }
    range_sq = block_sum_f64(range_sq, red);
    amax_sq = block_sum_f64(amax_sq, red);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) { lo = fminf(lo, __shfl_xor(lo, off)); hi = fmaxf(hi, __shfl_xor(hi, off)); }
    if ((threadIdx.x & 63) == 0) { redf[0][threadIdx.x >> 6] = lo; redf[1][threadIdx.x >> 6] = hi; }
    double sx = 0.0, sq = 0.0;
    for (int i = threadIdx.x; i < x_blocks; i += 256) { sx += xpart[2 * i]; sq += xpart[2 * i + 1]; }
    sx = block_sum_f64(sx, red);
    sq = block_sum_f64(sq, red);
    if (threadIdx.x != 0) return;
    lo = fminf(fminf(redf[0][0], redf[0][1]), fminf(redf[0][2], redf[0][3]));
    hi = fmaxf(fmaxf(redf[1][0], redf[1][1]), fmaxf(redf[1][2], redf[1][3]));
    const double mean = sx / x_count, var = fmax(sq / x_count - mean * mean, 0.0);
    const double g = stochastic ? (mean * mean + var) / 6.0 : var / 4.0;
    const double d = (double)N * (double)K, range = (double)hi - (double)lo, amax = fmax(fabs((double)lo), fabs((double)hi));
    const double q[3] = {7.0, 15.0, 255.0};
    for (int b = 0; b < 3; ++b) {
        omega[b] = 128.0 * range_sq / (q[b] * q[b]) * g;
        omega[4 + b] = d * (range / q[b]) * (range / q[b]) * g;
    }
    omega[3] = (double)K * amax_sq / (127.0 * 127.0) * g;
    omega[7] = d * (amax / 127.0) * (amax / 127.0) * g;
}

}  // namespace

int indicator_x_blocks(long n8) { return (int)std::min<long>(1024, std::max<long>(1, (n8 + 255) / 256)); }

size_t indicator_workspace_bytes(int N, long n8) { return (size_t)N * 4 * sizeof(float) + (size_t)indicator_x_blocks(n8) * 2 * sizeof(double) + 16; }

hipError_t launch_indicator(const void* w, int K, int N, const void* x, int M, int stochastic, double* omega, void* ws, hipStream_t s)
{
    const long n8 = (long)M * K / 8;
    const int xb = indicator_x_blocks(n8);
    double* xpart = static_cast<double*>(ws);                              // 16-byte aligned workspace: doubles first
    float* stats = reinterpret_cast<float*>(xpart + 2 * (size_t)xb);
    indicator_row_stats_kernel<<<(unsigned)((N + 3) / 4), 256, 0, s>>>(static_cast<const uint16_t*>(w), K, N, stats);
    indicator_x_sums_kernel<<<(unsigned)xb, 256, 0, s>>>(static_cast<const uint16_t*>(x), n8, xpart);
    indicator_finish_kernel<<<1, 256, 0, s>>>(stats, K, N, xpart, xb, (double)M * (double)K, stochastic, omega);
    return hipGetLastError();
}

}  // namespace lpq
