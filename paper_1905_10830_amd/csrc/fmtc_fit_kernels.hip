// Calibration statistics for the PCA basis (paper section 3: x ~ N(mu, Sigma);
// section 3.1 "Linear transform": covariance estimated on a small batch;
// "Quantization": dynamic range of the highest-variance channel).  Offline
// path: plain fp64 kernels, accumulated with fp64 atomics.
#include "fmtc_internal.h"

namespace fmtc {

__device__ __forceinline__ size_t elem_index(int layout, int64_t p, int c, int C, int64_t HW) {
    if (layout == FMTC_NHWC) return (size_t)p * (size_t)C + (size_t)c;
    int64_t n = p / HW, hw = p - n * HW;
    return ((size_t)n * (size_t)C + (size_t)c) * (size_t)HW + (size_t)hw;
}

// sum[c] += x[p][c] over the block's pixel range
__global__ __launch_bounds__(256) void k_fit_sum(const float* __restrict__ x, int64_t P, int C, int64_t HW,
                                                 int layout, int64_t px_per_block, double* __restrict__ sum) {
    const int64_t p0 = (int64_t)blockIdx.x * px_per_block;
    const int64_t p1 = (p0 + px_per_block < P) ? p0 + px_per_block : P;
    for (int c = threadIdx.x; c < C; c += 256) {
        double acc = 0.0;
        for (int64_t p = p0; p < p1; p++) acc += (double)x[elem_index(layout, p, c, C, HW)];
        atomicAdd(&sum[c], acc);
    }
}

// cov[i][j] += sum_p (x[p][i] - mean[i]) (x[p][j] - mean[j]); 16x16 outputs per block
__global__ __launch_bounds__(256) void k_fit_cov(const float* __restrict__ x, int64_t P, int C, int64_t HW,
                                                 int layout, int64_t px_per_block, const double* __restrict__ sum,
                                                 double* __restrict__ cov) {
    __shared__ double xi[16][17], xj[16][17];
    const int ti = threadIdx.x / 16, tj = threadIdx.x % 16;
    const int i0 = blockIdx.x * 16, j0 = blockIdx.y * 16;
    const int64_t p0 = (int64_t)blockIdx.z * px_per_block;
    const int64_t p1 = (p0 + px_per_block < P) ? p0 + px_per_block : P;
    const double Pd = (double)P;
    // this thread stages channel (i0 + tj) / (j0 + tj) of pixel slot ti
    const int ci = i0 + tj, cj = j0 + tj;
    const double mi = ci < C ? sum[ci] / Pd : 0.0;
    const double mj = cj < C ? sum[cj] / Pd : 0.0;
    double acc = 0.0;
    for (int64_t pb = p0; pb < p1; pb += 16) {
        int64_t p = pb + ti;
        xi[ti][tj] = (p < p1 && ci < C) ? (double)x[elem_index(layout, p, ci, C, HW)] - mi : 0.0;
        xj[ti][tj] = (p < p1 && cj < C) ? (double)x[elem_index(layout, p, cj, C, HW)] - mj : 0.0;
        __syncthreads();
#pragma unroll
        for (int q = 0; q < 16; q++) acc += xi[q][ti] * xj[q][tj];
        __syncthreads();
    }
    const int i = i0 + ti, j = j0 + tj;
    if (i < C && j < C) atomicAdd(&cov[(size_t)i * C + j], acc);
}

hipError_t launch_fit_moments(const float* d_x, int64_t N, int C, int64_t HW, int layout, double* d_sum,
                              double* d_cov, hipStream_t s) {
    const int64_t P = N * HW;
    int64_t blocks = (P + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    int64_t ppb = (P + blocks - 1) / blocks;
    blocks = (P + ppb - 1) / ppb;
    hipLaunchKernelGGL(k_fit_sum, dim3((unsigned)blocks), dim3(256), 0, s, d_x, P, C, HW, layout, ppb, d_sum);
    const unsigned tiles = (unsigned)((C + 15) / 16);
    int64_t splits = (P + 1023) / 1024;
    int64_t max_splits = 65536 / ((int64_t)tiles * tiles) + 1;
    if (splits > max_splits) splits = max_splits;
    if (splits > 1024) splits = 1024;
    int64_t ppb2 = (P + splits - 1) / splits;
    ppb2 = (ppb2 + 15) / 16 * 16;
    splits = (P + ppb2 - 1) / ppb2;
    hipLaunchKernelGGL(k_fit_cov, dim3(tiles, tiles, (unsigned)splits), dim3(256), 0, s, d_x, P, C, HW, layout, ppb2,
                       d_sum, d_cov);
    return hipGetLastError();
}

// amax = max_p | sum_c t0[c] (x[p][c] - mu[c]) |, fp64 accumulation in channel order
__global__ __launch_bounds__(256) void k_fit_range(const float* __restrict__ x, int64_t P, int C, int64_t HW,
                                                   int layout, const float* __restrict__ t0,
                                                   const float* __restrict__ mu,
                                                   unsigned long long* __restrict__ amax_bits) {
    double best = 0.0;
    for (int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x; p < P; p += (int64_t)gridDim.x * 256) {
        double acc = 0.0;
        for (int c = 0; c < C; c++) acc += (double)t0[c] * ((double)x[elem_index(layout, p, c, C, HW)] - (double)mu[c]);
        acc = fabs(acc);
        if (acc > best) best = acc;
    }
    // non-negative doubles order like their bit patterns
    if (best > 0.0) atomicMax(amax_bits, (unsigned long long)__double_as_longlong(best));
}

hipError_t launch_fit_range(const float* d_x, int64_t N, int C, int64_t HW, int layout, const float* d_t0,
                            const float* d_mu, double* d_amax, hipStream_t s) {
    const int64_t P = N * HW;
    int64_t blocks = (P + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(k_fit_range, dim3((unsigned)blocks), dim3(256), 0, s, d_x, P, C, HW, layout, d_t0, d_mu,
                       reinterpret_cast<unsigned long long*>(d_amax));
    return hipGetLastError();
}

}  // namespace fmtc
