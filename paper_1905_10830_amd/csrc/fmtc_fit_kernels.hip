// Calibration statistics for the PCA basis (paper section 3: x ~ N(mu, Sigma);
// section 3.1 "Linear transform": covariance estimated on a small batch;
// "Quantization": dynamic range of the highest-variance channel).  Offline
// path, fp64 throughout: channel sums, then the centred second moments on the
// fp64 matrix cores.
#include "fmtc_internal.h"

namespace fmtc {

__device__ __forceinline__ size_t elem_index(int layout, int64_t p, int c, int C, int64_t HW) {
    if (layout == FMTC_NHWC) return (size_t)p * (size_t)C + (size_t)c;
    int64_t n = p / HW, hw = p - n * HW;
    return ((size_t)n * (size_t)C + (size_t)c) * (size_t)HW + (size_t)hw;
}

// sum[c] += x[p][c] over the block's pixel range.  Thread t takes channel c0 + t % CB of every (256 / CB)-th pixel
// (CB = channels a block covers at a time: 64, 128 or 256), four loads in flight, fp64 sums; the threads of a
// channel are added in LDS and one fp64 atomic per channel and block goes out.
__global__ __launch_bounds__(256) void k_fit_sum(const float* __restrict__ x, int64_t P, int C, int64_t HW,
                                                 int layout, int64_t px_per_block, double* __restrict__ sum) {
    __shared__ double part[256];
    const int64_t p0 = (int64_t)blockIdx.x * px_per_block;
    const int64_t p1 = (p0 + px_per_block < P) ? p0 + px_per_block : P;
    const int CB = C <= 64 ? 64 : (C <= 128 ? 128 : 256);
    const int rows = 256 / CB, cl = threadIdx.x % CB, pr = threadIdx.x / CB;
    for (int c0 = 0; c0 < C; c0 += CB) {
        const int c = c0 + cl;
        double acc = 0.0;
        if (c < C) {
            int64_t p = p0 + pr;
            for (; p + 3 * rows < p1; p += 4 * rows) {
                const float v0 = x[elem_index(layout, p, c, C, HW)], v1 = x[elem_index(layout, p + rows, c, C, HW)];
                const float v2 = x[elem_index(layout, p + 2 * rows, c, C, HW)];
                const float v3 = x[elem_index(layout, p + 3 * rows, c, C, HW)];
                acc += ((double)v0 + (double)v1) + ((double)v2 + (double)v3);
            }
            for (; p < p1; p += rows) acc += (double)x[elem_index(layout, p, c, C, HW)];
        }
        part[threadIdx.x] = acc;
        __syncthreads();
        if (pr == 0 && c < C) {
            for (int r = 1; r < rows; r++) acc += part[r * CB + cl];
            atomicAdd(&sum[c], acc);
        }
        __syncthreads();
    }
}

// Centred second moments M[i][j] = sum_p (x[p][i] - mean[i]) (x[p][j] - mean[j]) as a symmetric rank-P update on the
// fp64 matrix cores (v_mfma_f64_16x16x4_f64: D[16x16] += A[16x4] B[4x16], fp64 in and out).  The pixel index is the
// contraction index: lane l holds A[l % 16][l / 16] = xc[p + l / 16][i0 + l % 16] and B[l / 16][l % 16] =
// xc[p + l / 16][j0 + l % 16] (xc = (double)x - mean), and of D the four entries D[4 r + l / 16][l % 16], r = 0..3.
// A workgroup owns a 64 x 64 block of M in the upper triangle of blocks (its four wavefronts 32 x 32 each, four
// accumulators of four doubles) over one slice of the pixels and writes its sums to its slice of `partial`
// ([splits][C][C]); off-diagonal blocks are written at both (i, j) and (j, i).  No atomics; k_fit_cov_reduce adds
// the slices in a fixed order.
typedef double doublex4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void k_fit_cov_mfma(const float* __restrict__ x, int64_t P, int C, int64_t HW,
                                                      int layout, int64_t px_per_split, int n_blocks,
                                                      const double* __restrict__ sum, double* __restrict__ partial) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // block pair (bi <= bj) number blockIdx.x of the upper triangle, rows of n_blocks, n_blocks - 1, ... entries
    int bi = 0, rest = (int)blockIdx.x;
    while (rest >= n_blocks - bi) {
        rest -= n_blocks - bi;
        bi++;
    }
    const int bj = bi + rest;
    const int ibase = bi * 64 + (wave >> 1) * 32, jbase = bj * 64 + (wave & 1) * 32;
    const int64_t p0 = (int64_t)blockIdx.y * px_per_split;
    const int64_t p1 = (p0 + px_per_split < P) ? p0 + px_per_split : P;
    const int col = lane & 15, krow = lane >> 4;
    const double Pd = (double)P;
    int ci[2], cj[2];
    double mi[2], mj[2];
#pragma unroll
    for (int t = 0; t < 2; t++) {
        ci[t] = ibase + 16 * t + col;
        cj[t] = jbase + 16 * t + col;
        mi[t] = ci[t] < C ? sum[ci[t]] / Pd : 0.0;
        mj[t] = cj[t] < C ? sum[cj[t]] / Pd : 0.0;
    }
    doublex4 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; a++)
#pragma unroll
        for (int b = 0; b < 2; b++) acc[a][b] = doublex4{0.0, 0.0, 0.0, 0.0};
    constexpr int U = 4;  // contraction steps (of four pixels) per turn: their loads are in flight together
    for (int64_t pb = p0; pb < p1; pb += 4 * U) {
        float va[U][2], vb[U][2];
#pragma unroll
        for (int u = 0; u < U; u++) {
            const int64_t pp = pb + 4 * u + krow;
            const bool ok = pp < p1;
#pragma unroll
            for (int t = 0; t < 2; t++) {
                va[u][t] = (ok && ci[t] < C) ? x[elem_index(layout, pp, ci[t], C, HW)] : 0.f;
                vb[u][t] = (ok && cj[t] < C) ? x[elem_index(layout, pp, cj[t], C, HW)] : 0.f;
            }
        }
#pragma unroll
        for (int u = 0; u < U; u++) {
            const bool ok = pb + 4 * u + krow < p1;
            double a[2], b[2];
#pragma unroll
            for (int t = 0; t < 2; t++) {
                a[t] = (ok && ci[t] < C) ? (double)va[u][t] - mi[t] : 0.0;
                b[t] = (ok && cj[t] < C) ? (double)vb[u][t] - mj[t] : 0.0;
            }
#pragma unroll
            for (int ta = 0; ta < 2; ta++)
#pragma unroll
                for (int tb = 0; tb < 2; tb++)
                    acc[ta][tb] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[ta], b[tb], acc[ta][tb], 0, 0, 0);
        }
    }
    double* out = partial + (size_t)blockIdx.y * (size_t)C * (size_t)C;
#pragma unroll
    for (int ta = 0; ta < 2; ta++)
#pragma unroll
        for (int tb = 0; tb < 2; tb++)
#pragma unroll
            for (int r = 0; r < 4; r++) {
                const int i = ibase + 16 * ta + 4 * r + krow, j = jbase + 16 * tb + col;
                if (i < C && j < C) {
                    out[(size_t)i * C + j] = acc[ta][tb][r];
                    if (bi != bj) out[(size_t)j * C + i] = acc[ta][tb][r];
                }
            }
}

// cov[e] = sum over the slices of partial[slice][e], slices in ascending order
__global__ __launch_bounds__(256) void k_fit_cov_reduce(const double* __restrict__ partial, int splits, size_t n,
                                                        double* __restrict__ cov) {
    const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= n) return;
    double acc = 0.0;
    int q = 0;
    for (; q + 3 < splits; q += 4) {  // four loads in flight; the sum stays in ascending order
        const double a0 = partial[(size_t)q * n + e], a1 = partial[(size_t)(q + 1) * n + e];
        const double a2 = partial[(size_t)(q + 2) * n + e], a3 = partial[(size_t)(q + 3) * n + e];
        acc = (((acc + a0) + a1) + a2) + a3;
    }
    for (; q < splits; q++) acc += partial[(size_t)q * n + e];
    cov[e] = acc;
}

// Slices of the pixels for the second moments (each costs C * C doubles of scratch): enough workgroups to fill the
// device, at least 64 pixels a slice, at most 64 MB of scratch.
static void fit_cov_plan(int64_t P, int C, int* n_blocks, int64_t* splits, int64_t* px_per_split) {
    const int nb = (C + 63) / 64;
    const int64_t pairs = (int64_t)nb * (nb + 1) / 2;
    int64_t sp = (1024 + pairs - 1) / pairs;
    const int64_t by_px = (P + 63) / 64;
    if (sp > by_px) sp = by_px;
    const int64_t by_mem = (64ll << 20) / ((int64_t)C * C * 8);
    if (sp > by_mem) sp = by_mem;
    if (sp < 1) sp = 1;
    int64_t pps = (P + sp - 1) / sp;
    pps = (pps + 15) / 16 * 16;
    *n_blocks = nb;
    *px_per_split = pps;
    *splits = (P + pps - 1) / pps;
}

size_t fit_moments_scratch_bytes(int64_t P, int C) {
    int nb;
    int64_t splits, pps;
    fit_cov_plan(P, C, &nb, &splits, &pps);
    return (size_t)splits * (size_t)C * (size_t)C * sizeof(double);
}

hipError_t launch_fit_moments(const float* d_x, int64_t N, int C, int64_t HW, int layout, double* d_sum,
                              double* d_cov, double* d_scratch, hipStream_t s) {
    const int64_t P = N * HW;
    int64_t blocks = (P + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    int64_t ppb = (P + blocks - 1) / blocks;
    blocks = (P + ppb - 1) / ppb;
    hipLaunchKernelGGL(k_fit_sum, dim3((unsigned)blocks), dim3(256), 0, s, d_x, P, C, HW, layout, ppb, d_sum);
    int nb;
    int64_t splits, pps;
    fit_cov_plan(P, C, &nb, &splits, &pps);
    hipLaunchKernelGGL(k_fit_cov_mfma, dim3((unsigned)(nb * (nb + 1) / 2), (unsigned)splits), dim3(256), 0, s, d_x, P, C,
                       HW, layout, pps, nb, d_sum, d_scratch);
    const size_t n = (size_t)C * (size_t)C;
    hipLaunchKernelGGL(k_fit_cov_reduce, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, d_scratch, (int)splits, n,
                       d_cov);
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
