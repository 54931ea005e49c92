// Encoder front end: y = T(x - mu), uniform quantizer, symbol histogram
// (paper section 3; section 3.1 "Linear transform", "Quantization",
// "Variable length coding" for the statistics).
//
// The projection of all pixels is one dense contraction [C x C] . [C x P]; it
// runs on the fp32 matrix cores (v_mfma_f32_32x32x2_f32).  Per workgroup:
// 4 wavefronts = WK coefficient tiles (32 each) x WP pixel groups; the basis
// tile is read from its pre-packed operand order straight into registers, the
// activations go through LDS (coalesced global reads, transposed so that a
// wavefront reads 32 consecutive pixels of one channel).  The quantized tile is
// staged in LDS and leaves as whole rows of symbols.
#include "fmtc_internal.h"

namespace fmtc {

typedef float floatx16 __attribute__((ext_vector_type(16)));

__global__ void k_clear(uint32_t* __restrict__ w, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) w[i] = 0u;
}

hipError_t launch_clear(uint32_t* d_words, size_t n_words, hipStream_t s) {
    if (n_words == 0) return hipSuccess;
    unsigned blocks = (unsigned)((n_words + 255) / 256);
    ProfScope prof(K_CLEAR, s);
    hipLaunchKernelGGL(k_clear, dim3(blocks), dim3(256), 0, s, d_words, n_words);
    return hipGetLastError();
}

// WK: wavefronts along the coefficient axis (1, 2 or 4); MT: 32-pixel tiles per
// wavefront; LAYOUT: FMTC_NHWC / FMTC_NCHW; VEC: C % 4 == 0 (16-byte loads of
// channels-last rows and 4-byte symbol stores are aligned).
template <int WK, int MT, int LAYOUT, bool VEC>
__global__ __launch_bounds__(256) void k_project_quantize(const float* __restrict__ x,
                                                          const float* __restrict__ Apk,
                                                          const float* __restrict__ mu,
                                                          const float* __restrict__ Trow, int64_t P, int64_t HW,
                                                          int C, int ncs, float inv_delta, float delta, float tau,
                                                          int bits,
                                                          uint8_t* __restrict__ syms,
                                                          uint32_t* __restrict__ hist_copies) {
    constexpr int WP = 4 / WK;
    constexpr int PT = WP * MT * 32;  // pixels per workgroup
    constexpr int S = PT + 2;         // LDS row stride in floats: conflict-free writes (4S = 8 mod 64) and reads (16S = 32 mod 64)
    constexpr int NLV = PT / 32;      // float4 loads per thread and channel step (channels-last, VEC)
    constexpr int NLS = PT / 8;       // scalar loads per thread and channel step
    constexpr int RSW = WK * 8 + 1;   // staging row stride in words

    __shared__ float xs[2][32 * S];
    __shared__ uint32_t lhist[256];
    static_assert(sizeof(float) * 2 * 32 * S >= sizeof(uint32_t) * PT * RSW, "staging tile must fit");

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wk = wave % WK, wp = wave / WK;
    const int half = lane >> 5, l32 = lane & 31;
    const int64_t px0 = (int64_t)blockIdx.x * PT;
    const int kt = blockIdx.y * WK + wk;
    const bool kt_valid = kt < ncs;

    lhist[tid] = 0u;

    // ---- per-thread load coordinates (fixed over the channel steps) ----
    float4 xv[VEC && LAYOUT == FMTC_NHWC ? NLV : 1];
    float xsc[VEC && LAYOUT == FMTC_NHWC ? 1 : NLS];
    int64_t nchw_base = 0;
    bool nchw_ok = false;
    if constexpr (LAYOUT == FMTC_NCHW) {
        int64_t p = px0 + (tid % PT);
        nchw_ok = p < P;
        if (nchw_ok) {
            int64_t n = p / HW, hw = p - n * HW;
            nchw_base = n * (int64_t)C * HW + hw;
        }
    }

    auto load_step = [&](int cs) {
        if constexpr (LAYOUT == FMTC_NHWC && VEC) {
#pragma unroll
            for (int j = 0; j < NLV; j++) {
                int pxl = (tid >> 3) + 32 * j;
                int c = cs * 32 + 4 * (tid & 7);
                int64_t px = px0 + pxl;
                xv[j] = (px < P && c < C) ? *reinterpret_cast<const float4*>(x + px * C + c) : make_float4(0, 0, 0, 0);
            }
        } else if constexpr (LAYOUT == FMTC_NHWC) {
#pragma unroll
            for (int j = 0; j < NLS; j++) {
                int pxl = (tid >> 5) + 8 * j;
                int c = cs * 32 + (tid & 31);
                int64_t px = px0 + pxl;
                xsc[j] = (px < P && c < C) ? x[px * C + c] : 0.f;
            }
        } else {
#pragma unroll
            for (int j = 0; j < NLS; j++) {
                int c = cs * 32 + tid / PT + (256 / PT) * j;
                xsc[j] = (nchw_ok && c < C) ? x[nchw_base + (int64_t)c * HW] : 0.f;
            }
        }
    };
    auto store_step = [&](int cs, float* dst) {
        if constexpr (LAYOUT == FMTC_NHWC && VEC) {
            int cl = 4 * (tid & 7);
            float4 m = *reinterpret_cast<const float4*>(mu + cs * 32 + cl);
#pragma unroll
            for (int j = 0; j < NLV; j++) {
                int pxl = (tid >> 3) + 32 * j;
                dst[(cl + 0) * S + pxl] = xv[j].x - m.x;
                dst[(cl + 1) * S + pxl] = xv[j].y - m.y;
                dst[(cl + 2) * S + pxl] = xv[j].z - m.z;
                dst[(cl + 3) * S + pxl] = xv[j].w - m.w;
            }
        } else if constexpr (LAYOUT == FMTC_NHWC) {
            int cl = tid & 31;
            float m = mu[cs * 32 + cl];
#pragma unroll
            for (int j = 0; j < NLS; j++) dst[cl * S + (tid >> 5) + 8 * j] = xsc[j] - m;
        } else {
#pragma unroll
            for (int j = 0; j < NLS; j++) {
                int cl = tid / PT + (256 / PT) * j;
                dst[cl * S + (tid % PT)] = xsc[j] - mu[cs * 32 + cl];
            }
        }
    };
    auto load_a = [&](int cs, float4* a) {
        const float4* src = reinterpret_cast<const float4*>(Apk + ((size_t)(kt * ncs + cs) * 64 + lane) * 16);
#pragma unroll
        for (int j = 0; j < 4; j++) a[j] = kt_valid ? src[j] : make_float4(0, 0, 0, 0);
    };

    floatx16 acc[MT];
#pragma unroll
    for (int m = 0; m < MT; m++)
#pragma unroll
        for (int r = 0; r < 16; r++) acc[m][r] = 0.f;

    float4 a_cur[4], a_nxt[4];
    load_step(0);
    load_a(0, a_cur);
    store_step(0, xs[0]);
    __syncthreads();

    for (int cs = 0; cs < ncs; cs++) {
        const bool more = cs + 1 < ncs;
        if (more) {
            load_step(cs + 1);
            load_a(cs + 1, a_nxt);
        }
        if (kt_valid) {
            const float* src = xs[cs & 1] + (16 * half) * S + wp * MT * 32 + l32;
#pragma unroll
            for (int s = 0; s < 16; s++) {
                float a = reinterpret_cast<const float*>(a_cur)[s];
#pragma unroll
                for (int m = 0; m < MT; m++) {
                    float b = src[s * S + m * 32];
                    acc[m] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[m], 0, 0, 0);
                }
            }
        }
        if (more) {
            store_step(cs + 1, xs[(cs + 1) & 1]);
#pragma unroll
            for (int j = 0; j < 4; j++) a_cur[j] = a_nxt[j];
        }
        __syncthreads();
    }

    // ---- quantize ----
    // accumulator r of lane l holds coefficient kt*32 + 8*(r/4) + 4*(l/32) + r%4 of pixel l%32
    uint32_t* st = reinterpret_cast<uint32_t*>(&xs[0][0]);
    const int zero_sym = 1 << (bits - 1);
    const float lo = (float)(-zero_sym), hi = (float)(zero_sym - 1);
    uint32_t words[MT][4];
    uint32_t near_mask = 0;  // bit m*16 + r: the fp32 value is too close to a rounding boundary to be trusted
    if (kt_valid) {
#pragma unroll
        for (int m = 0; m < MT; m++) {
            const bool px_ok = px0 + (wp * MT + m) * 32 + l32 < P;
#pragma unroll
            for (int g = 0; g < 4; g++) {
                const int k = kt * 32 + 8 * g + 4 * half;
                uint32_t word = 0;
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    float t = acc[m][4 * g + i] * inv_delta;
                    float q = __builtin_rintf(t);  // round half to even
                    bool near = fabsf(t - q) > 0.5f - tau;
                    q = fminf(fmaxf(q, lo), hi);
                    word |= (uint32_t)((int)q + zero_sym) << (8 * i);
                    if (near && px_ok && (k + i) < C) near_mask |= 1u << (m * 16 + 4 * g + i);
                }
                words[m][g] = word;
            }
        }
        // ---- exact decision for the flagged values: the whole wavefront recomputes y in fp64 ----
        // (same arithmetic as the definition: sum of T[k][c] * (x[c] - mu[c]), divided by the step)
        unsigned long long pending = __ballot(near_mask != 0);
        while (pending) {
            const int L = __ffsll((long long)pending) - 1;
            const uint32_t fm = (uint32_t)__builtin_amdgcn_readlane((int)near_mask, L);
            const int v = __ffs((int)fm) - 1;
            const int m = v >> 4, r = v & 15;
            const int k = kt * 32 + 8 * (r >> 2) + 4 * (L >> 5) + (r & 3);
            const int64_t px = px0 + (wp * MT + m) * 32 + (L & 31);
            int64_t xbase, xstride;
            if constexpr (LAYOUT == FMTC_NHWC) {
                xbase = px * C;
                xstride = 1;
            } else {
                int64_t n = px / HW;
                xbase = n * (int64_t)C * HW + (px - n * HW);
                xstride = HW;
            }
            double part = 0.0;
            for (int c = lane; c < C; c += 64)
                part += (double)Trow[(size_t)k * C + c] * ((double)x[xbase + c * xstride] - (double)mu[c]);
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) part += __shfl_xor(part, o, 64);
            double qd = rint(part / (double)delta);
            qd = fmin(fmax(qd, (double)lo), (double)hi);
            const uint32_t sfix = (uint32_t)((int)qd + zero_sym);
            if (lane == L) {
#pragma unroll
                for (int mm = 0; mm < MT; mm++)
#pragma unroll
                    for (int g = 0; g < 4; g++)
                        if (mm == m && g == (r >> 2))
                            words[mm][g] = (words[mm][g] & ~(0xffu << (8 * (r & 3)))) | (sfix << (8 * (r & 3)));
                near_mask &= ~(1u << v);
            }
            pending = __ballot(near_mask != 0);
        }
        // ---- count and stage ----
        uint32_t zero_count = 0;
#pragma unroll
        for (int m = 0; m < MT; m++) {
            const int pxl = (wp * MT + m) * 32 + l32;
            const bool px_ok = px0 + pxl < P;
#pragma unroll
            for (int g = 0; g < 4; g++) {
                const int k = kt * 32 + 8 * g + 4 * half;
                const uint32_t word = words[m][g];
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    int sy = (int)((word >> (8 * i)) & 255u);
                    bool ok = px_ok && (k + i) < C;
                    zero_count += (uint32_t)__popcll(__ballot(ok && sy == zero_sym));
                    if (ok && sy != zero_sym) atomicAdd(&lhist[sy], 1u);
                }
                st[pxl * RSW + wk * 8 + 2 * g + half] = word;
            }
        }
        if (lane == 0 && zero_count) atomicAdd(&lhist[zero_sym], zero_count);
    }
    __syncthreads();

    // ---- symbols leave as rows of WK*32 bytes per pixel ----
    const int kbase = blockIdx.y * WK * 32;
    for (int idx = tid; idx < PT * WK * 8; idx += 256) {
        int row = idx / (WK * 8), col = idx % (WK * 8);
        int64_t px = px0 + row;
        int k = kbase + 4 * col;
        if (px < P && k < C) {
            uint32_t word = st[row * RSW + col];
            uint8_t* dst = syms + px * C + k;
            if constexpr (VEC) {
                *reinterpret_cast<uint32_t*>(dst) = word;
            } else {
                for (int i = 0; i < 4 && k + i < C; i++) dst[i] = (uint8_t)(word >> (8 * i));
            }
        }
    }
    uint32_t hcount = lhist[tid];
    if (hcount) {
        unsigned copy = (blockIdx.x + blockIdx.y * gridDim.x) % kHistCopies;
        atomicAdd(&hist_copies[copy * 256 + tid], hcount);
    }
}

template <int WK, int MT>
static hipError_t launch_pq(const BasisDevice& b, const float* d_x, int64_t P, int64_t HW, int layout, float delta,
                            int bits, uint8_t* d_syms, uint32_t* d_hist_copies, hipStream_t s) {
    const float inv_delta = (float)(1.0 / (double)delta);
    // fp32 accumulation of C terms is off by about sqrt(C) * 2^-24 * |x - mu| / delta steps; values within
    // tau (a few times that) of a rounding boundary are decided in fp64 instead
    float tau = 8.f * sqrtf((float)b.Cpad) * 5.9604645e-8f * (float)(1 << (bits - 1));
    tau = fminf(fmaxf(tau, 1.f / 8192.f), 1.f / 128.f);
    constexpr int PT = (4 / WK) * MT * 32;
    const int ncs = b.Cpad / 32;
    dim3 grid((unsigned)((P + PT - 1) / PT), (unsigned)((ncs + WK - 1) / WK));
    const bool vec = (b.C % 4) == 0;
    ProfScope prof(K_PROJECT, s);
#define FMTC_PQ(LAY, VEC)                                                                                      \
    hipLaunchKernelGGL((k_project_quantize<WK, MT, LAY, VEC>), grid, dim3(256), 0, s, d_x, b.fwd, b.mu, b.T, P, \
                       HW, b.C, ncs, inv_delta, delta, tau, bits, d_syms, d_hist_copies)
    if (layout == FMTC_NHWC) {
        if (vec) FMTC_PQ(FMTC_NHWC, true);
        else FMTC_PQ(FMTC_NHWC, false);
    } else {
        if (vec) FMTC_PQ(FMTC_NCHW, true);
        else FMTC_PQ(FMTC_NCHW, false);
    }
#undef FMTC_PQ
    return hipGetLastError();
}

hipError_t launch_project_quantize(const BasisDevice& b, const float* d_x, int64_t N, int64_t HW, int layout,
                                   float delta, int bits, uint8_t* d_syms, uint32_t* d_hist_copies,
                                   hipStream_t s) {
    const int64_t P = N * HW;
    const int nkt = b.Cpad / 32;
    if (nkt == 1) return launch_pq<1, 1>(b, d_x, P, HW, layout, delta, bits, d_syms, d_hist_copies, s);
    if (nkt == 2) return launch_pq<2, 1>(b, d_x, P, HW, layout, delta, bits, d_syms, d_hist_copies, s);
    return launch_pq<4, 2>(b, d_x, P, HW, layout, delta, bits, d_syms, d_hist_copies, s);
}

// Histogram of given symbols (staged coder entry point).  counters[0] receives
// the number of symbols outside the alphabet (must stay 0).
__global__ __launch_bounds__(256) void k_histogram(const uint8_t* __restrict__ syms, uint64_t V, int bits,
                                                   uint32_t* __restrict__ hist_copies,
                                                   uint32_t* __restrict__ counters) {
    __shared__ uint32_t lhist[256];
    lhist[threadIdx.x] = 0u;
    __syncthreads();
    const unsigned K = 1u << bits;
    uint32_t bad = 0;
    for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < V; i += (uint64_t)gridDim.x * 256) {
        unsigned s = syms[i];
        if (s < K) atomicAdd(&lhist[s], 1u);
        else bad++;
    }
    __syncthreads();
    uint32_t h = lhist[threadIdx.x];
    if (h) atomicAdd(&hist_copies[(blockIdx.x % kHistCopies) * 256 + threadIdx.x], h);
    if (bad) atomicAdd(&counters[0], bad);
}

hipError_t launch_histogram(const uint8_t* d_syms, uint64_t V, int bits, uint32_t* d_hist_copies,
                            uint32_t* d_counters, hipStream_t s) {
    uint64_t want = (V + 256 * 16 - 1) / (256 * 16);
    unsigned blocks = (unsigned)(want < 1 ? 1 : (want > 2048 ? 2048 : want));
    ProfScope prof(K_HISTOGRAM, s);
    hipLaunchKernelGGL(k_histogram, dim3(blocks), dim3(256), 0, s, d_syms, V, bits, d_hist_copies, d_counters);
    return hipGetLastError();
}

}  // namespace fmtc
