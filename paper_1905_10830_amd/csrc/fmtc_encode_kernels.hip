// Encoder front end: y = T(x - mu), uniform quantizer, symbol histogram
// (paper section 3; section 3.1 "Linear transform", "Quantization",
// "Variable length coding" for the statistics).
//
// The projection of all pixels is one dense contraction [C x C] . [C x P].  It
// runs on the f16 matrix cores (v_mfma_f32_32x32x16_f16) with every fp32 operand
// split into two f16 parts, which is as accurate as the fp32 matrix instruction
// and several times as fast; values that land too close to a rounding boundary
// for the fast pass to decide are recomputed in fp64 by the wavefront.  Two
// kernels: one wavefront per 32 pixels with the basis in LDS (up to 160
// channels), and a workgroup tile in LDS with the basis streamed from L2 (wider).
#include <atomic>
#include <type_traits>

#include "fmtc_device.h"
#include "fmtc_internal.h"
#include "fmtc_pack_device.h"

namespace fmtc {

typedef float floatx16 __attribute__((ext_vector_type(16)));

// ---------------------------------------------------------------------------
// Wide tensors (more than 160 channels after padding to 32).  The contraction is the same f16
// split as in the narrow-tensor kernel below (three v_mfma_f32_32x32x16_f16 per 16 channels,
// see there), but a pixel's channels no longer fit a wavefront's registers: the workgroup
// (8 wavefronts) first brings a tile of PT pixels, all channels, into LDS -- coalesced global
// reads, mean removed and split into the two f16 parts on the way, rows padded by 16 bytes so
// that the 16-byte operand reads of 8 neighbouring pixels cover all banks -- then its
// wavefronts share out the work units (coefficient tile, 32-pixel group) of the workgroup's
// coefficient range [kt0, kt0 + ktg) without further barriers, the four wavefronts of a round
// taking the pixel groups of one coefficient tile so that they read the same part of the
// basis, which streams from L2 in operand order one step ahead of its use.  Values too close
// to a rounding boundary are recomputed in fp64; the quantized tile is staged in LDS and
// leaves as whole rows of symbols.
// PT: pixels per workgroup; LAYOUT: FMTC_NHWC / FMTC_NCHW; VEC: C % 4 == 0 (16-byte loads of
// channels-last rows and 4-byte symbol stores are aligned).
// ---------------------------------------------------------------------------
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));
typedef _Float16 halfx4 __attribute__((ext_vector_type(4)));

struct WideParams {
    const float* x;
    const uint16_t* basis16;  // fwd16 packing
    const float* mu;          // [Cpad]
    const float* Trow;        // [C][C] row major, for the exact decisions
    int64_t P, HW;
    int C, ncs, kt_per_group, bits;
    float inv_delta, delta, kappa, tau_min;
    int64_t px_tiles;
    uint8_t* syms;
    uint32_t* hist_parts;
    CoderCtrl* ctrl;
    unsigned long long* lookback;
    uint32_t n_groups;
};

constexpr int kWideThreads = 512;

template <int PT, int LAYOUT, bool VEC>
__global__ __launch_bounds__(kWideThreads) void k_project_quantize_wide(WideParams p) {
    extern __shared__ __align__(16) uint8_t dyn_lds[];
    __shared__ uint32_t lhist[256];
    __shared__ float s_n2[PT];  // |x - mu|^2 of every pixel of the tile
    zero_coder_scratch(p.ctrl, p.lookback, p.n_groups);

    const int C = p.C, ncs = p.ncs;
    const int Cpad = ncs * 32, NJ = ncs * 2;
    const int RSH = Cpad + 8;  // pixel row stride in halves
    const int kt0 = blockIdx.y * p.kt_per_group;
    const int ktg = (ncs - kt0 < p.kt_per_group) ? ncs - kt0 : p.kt_per_group;
    const int RSW = p.kt_per_group * 8 + 1;  // staging row stride in words
    _Float16* xh = reinterpret_cast<_Float16*>(dyn_lds);
    _Float16* xl = xh + (size_t)PT * RSH;
    uint32_t* st = reinterpret_cast<uint32_t*>(xl + (size_t)PT * RSH);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, l32 = lane & 31;

    if (tid < 256) lhist[tid] = 0u;
    const int zero_sym = 1 << (p.bits - 1);
    const float lo = (float)(-zero_sym), hi = (float)(zero_sym - 1);
    const float inv_delta = p.inv_delta, inv_delta_lo = p.inv_delta * (1.f / 2048.f);

    // the two f16 parts of one value (clamped to what f16 holds: a pixel with such a value is decided exactly)
    auto split = [](float v, _Float16& vh, _Float16& vl) {
        v = __builtin_amdgcn_fmed3f(v, -60000.f, 60000.f);
        vh = (_Float16)v;
        vl = (_Float16)((v - (float)vh) * 2048.f);
    };

    // the workgroup walks over pixel tiles; its histogram accumulates in LDS and leaves once at the end
    for (int64_t tile = blockIdx.x; tile < p.px_tiles; tile += gridDim.x) {
        const int64_t px0 = tile * PT;
        if (tid < PT) s_n2[tid] = 0.f;
        __syncthreads();  // also: the previous tile's staging rows have left

        // ---- the pixel tile, mean removed, split, as xh / xl [pixel][channel] ----
        if constexpr (LAYOUT == FMTC_NHWC && VEC) {
            const int n4 = PT * (C / 4);  // the tile is one contiguous run of PT*C floats
            const float* src = p.x + px0 * C;
            const int64_t lim = (p.P - px0) * C;  // floats of the tile that exist
            constexpr int B = 8;  // loads in flight per thread
            for (int idx0 = tid; idx0 < n4; idx0 += B * kWideThreads) {
                float4 v[B];
#pragma unroll
                for (int b = 0; b < B; b++) {
                    const int f = 4 * (idx0 + b * kWideThreads);
                    v[b] = (idx0 + b * kWideThreads < n4 && f < lim) ? *reinterpret_cast<const float4*>(src + f)
                                                                     : make_float4(0, 0, 0, 0);
                }
#pragma unroll
                for (int b = 0; b < B; b++) {
                    const int idx = idx0 + b * kWideThreads;
                    if (idx < n4) {
                        const int f = 4 * idx;
                        const int pxl = f / C, c = f - pxl * C;
                        const float4 m = *reinterpret_cast<const float4*>(p.mu + c);
                        const float d[4] = {v[b].x - m.x, v[b].y - m.y, v[b].z - m.z, v[b].w - m.w};
                        halfx4 vh, vl;
                        float n2 = 0.f;
#pragma unroll
                        for (int i = 0; i < 4; i++) {
                            _Float16 a, bb;
                            split(d[i], a, bb);
                            vh[i] = a;
                            vl[i] = bb;
                            n2 = __builtin_fmaf(d[i], d[i], n2);
                        }
                        *reinterpret_cast<halfx4*>(xh + pxl * RSH + c) = vh;
                        *reinterpret_cast<halfx4*>(xl + pxl * RSH + c) = vl;
                        atomicAdd(&s_n2[pxl], n2);
                    }
                }
            }
        } else if constexpr (LAYOUT == FMTC_NHWC) {
            const int n1 = PT * C;
            const float* src = p.x + px0 * C;
            for (int idx = tid; idx < n1; idx += kWideThreads) {
                const int pxl = idx / C, c = idx - pxl * C;
                const float d = ((px0 + pxl < p.P) ? src[idx] : 0.f) - p.mu[c];
                _Float16 a, b;
                split(d, a, b);
                xh[pxl * RSH + c] = a;
                xl[pxl * RSH + c] = b;
                atomicAdd(&s_n2[pxl], d * d);
            }
        } else {
            const int pxl = tid % PT;
            const int64_t px = px0 + pxl;
            const bool ok = px < p.P;
            int64_t base = 0;
            if (ok) {
                const int64_t n = px / p.HW;
                base = n * (int64_t)C * p.HW + (px - n * p.HW);
            }
            float n2 = 0.f;
            for (int c = tid / PT; c < C; c += kWideThreads / PT) {
                const float d = (ok ? p.x[base + (int64_t)c * p.HW] : 0.f) - p.mu[c];
                _Float16 a, b;
                split(d, a, b);
                xh[pxl * RSH + c] = a;
                xl[pxl * RSH + c] = b;
                n2 = __builtin_fmaf(d, d, n2);
            }
            atomicAdd(&s_n2[pxl], n2);
        }
        if (Cpad > C) {  // padding channels meet zero basis entries; they must still be finite
            const int padw = Cpad - C;
            for (int idx = tid; idx < PT * padw; idx += kWideThreads) {
                const int pxl = idx / padw, c = C + (idx - pxl * padw);
                xh[pxl * RSH + c] = (_Float16)0.f;
                xl[pxl * RSH + c] = (_Float16)0.f;
            }
        }
        __syncthreads();

        constexpr int PG = PT / 32;  // pixel groups per workgroup
        const int nunits = ktg * PG;
        for (int u = wave; u < nunits; u += kWideThreads / 64) {
            const int pg = u % PG, ktl = u / PG;
            const int kt = kt0 + ktl;
            const int pxl = pg * 32 + l32;
            const bool px_ok = px0 + pxl < p.P;
            floatx16 am, ac;
#pragma unroll
            for (int r = 0; r < 16; r++) { am[r] = 0.f; ac[r] = 0.f; }

            // (kt, j): the 64 lanes' hi parts, then their lo parts, 16 bytes per lane each; the basis comes from L2
            // (the wavefronts of a round read the same part of it), one step ahead of its use
            const uint4* asrc = reinterpret_cast<const uint4*>(p.basis16) + (size_t)kt * NJ * 2 * 64 + lane;
            uint4 th4 = asrc[0], tl4 = asrc[64];
            const _Float16* bh = xh + pxl * RSH + 8 * half;
            const _Float16* bl = xl + pxl * RSH + 8 * half;
            for (int jj = 0; jj < NJ; jj++) {
                uint4 nh4 = th4, nl4 = tl4;
                if (jj + 1 < NJ) {
                    nh4 = asrc[(size_t)(2 * jj + 2) * 64];
                    nl4 = asrc[(size_t)(2 * jj + 3) * 64];
                }
                const halfx8 th = __builtin_bit_cast(halfx8, th4), tl = __builtin_bit_cast(halfx8, tl4);
                const halfx8 xh8 = *reinterpret_cast<const halfx8*>(bh + 16 * jj);
                const halfx8 xl8 = *reinterpret_cast<const halfx8*>(bl + 16 * jj);
                am = __builtin_amdgcn_mfma_f32_32x32x16_f16(th, xh8, am, 0, 0, 0);
                ac = __builtin_amdgcn_mfma_f32_32x32x16_f16(th, xl8, ac, 0, 0, 0);
                ac = __builtin_amdgcn_mfma_f32_32x32x16_f16(tl, xh8, ac, 0, 0, 0);
                th4 = nh4;
                tl4 = nl4;
            }

            // ---- quantize ----
            // accumulator r = 4g + i of lane (pixel, h) is coefficient kt*32 + 16h + 4g + i of the pixel
            const float n2 = s_n2[pxl];
            const bool force = !(n2 < 1.0e9f);  // too large for f16, or not finite: every coefficient decided exactly
            const float tau = fminf(fmaxf(p.kappa * __builtin_sqrtf(n2), p.tau_min), 0.125f);
            const float near_limit = force ? -1.f : 0.5f - tau;
            const int k0 = kt * 32 + 16 * half;
            uint32_t words[4];
            uint32_t near_mask = 0;  // bit r: the fast value is too close to a rounding boundary to be trusted
#pragma unroll
            for (int g = 0; g < 4; g++) {
                uint32_t word = 0;
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    const float t = __builtin_fmaf(ac[4 * g + i], inv_delta_lo, am[4 * g + i] * inv_delta);
                    float q = __builtin_rintf(t);  // round half to even
                    const bool near = !(fabsf(t - q) <= near_limit);
                    q = __builtin_amdgcn_fmed3f(q, lo, hi);
                    word |= (uint32_t)((int)q + zero_sym) << (8 * i);
                    if (near && px_ok && (k0 + 4 * g + i) < C) near_mask |= 1u << (4 * g + i);
                }
                words[g] = word;
            }
            // ---- exact decision for the flagged values: fp64 recomputation, four values per round ----
            // (same arithmetic as the definition: sum of T[k][c] * (x[c] - mu[c]), divided by the step).
            // Each 16-lane group of the wavefront takes one flagged value, so the loads of four values overlap.
            unsigned long long pending = __ballot(near_mask != 0);
            while (pending) {
                int Ls[4];
                unsigned long long pm = pending;
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    Ls[q] = pm ? (__ffsll((long long)pm) - 1) : -1;
                    pm &= pm - 1;
                }
                const int grp = lane >> 4;
                const int Lq = grp == 0 ? Ls[0] : (grp == 1 ? Ls[1] : (grp == 2 ? Ls[2] : Ls[3]));
                const bool active = Lq >= 0;
                const uint32_t fm = (uint32_t)__shfl((int)near_mask, active ? Lq : 0, 64);
                const int r = active ? (__ffs((int)fm) - 1) : 0;
                const int k = kt * 32 + 16 * (Lq >> 5) + r;
                const int64_t px = px0 + pg * 32 + (Lq & 31);
                double part = 0.0;
                if (active) {
                    int64_t xbase, xstride;
                    if constexpr (LAYOUT == FMTC_NHWC) {
                        xbase = px * C;
                        xstride = 1;
                    } else {
                        const int64_t n = px / p.HW;
                        xbase = n * (int64_t)C * p.HW + (px - n * p.HW);
                        xstride = p.HW;
                    }
#pragma unroll 8  // independent loads of eight terms in flight together: the loop is all latency
                    for (int c = lane & 15; c < C; c += 16)
                        part += (double)p.Trow[(size_t)k * C + c] * ((double)p.x[xbase + c * xstride] - (double)p.mu[c]);
                }
#pragma unroll
                for (int o = 8; o > 0; o >>= 1) part += __shfl_xor(part, o, 64);  // stays inside the 16-lane group
                double qd = rint(part / (double)p.delta);
                qd = fmin(fmax(qd, (double)lo), (double)hi);
                const int sfix = (int)qd + zero_sym;
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    const int rq = __shfl(r, 16 * q, 64);
                    const int sq = __shfl(sfix, 16 * q, 64);
                    if (lane == Ls[q]) {
#pragma unroll
                        for (int g = 0; g < 4; g++)
                            if (g == (rq >> 2))
                                words[g] = (words[g] & ~(0xffu << (8 * (rq & 3)))) | ((uint32_t)sq << (8 * (rq & 3)));
                        near_mask &= ~(1u << rq);
                    }
                }
                pending = __ballot(near_mask != 0);
            }
            // ---- count and stage ----
            // zero-level symbols (the bulk) are counted with byte arithmetic, the others with LDS atomics
            uint32_t zero_count = 0;
            const uint32_t zero4 = (uint32_t)zero_sym * 0x01010101u;
#pragma unroll
            for (int g = 0; g < 4; g++) {
                const int k = k0 + 4 * g;
                const uint32_t word = words[g];
                // 0x80 in every byte of the word that is a valid coefficient
                const int nvalid = !px_ok ? 0 : (C - k >= 4 ? 4 : (C - k > 0 ? C - k : 0));
                const uint32_t vmask = nvalid == 4 ? 0x80808080u : (0x80808080u >> (8 * (4 - nvalid))) * (nvalid != 0);
                const uint32_t xz = word ^ zero4;
                uint32_t t = (xz & 0x7f7f7f7fu) + 0x7f7f7f7fu;
                t = ~(t | xz | 0x7f7f7f7fu);  // 0x80 where the byte equals the zero level
                zero_count += (uint32_t)__popc(t & vmask);
                uint32_t nz = ~t & vmask;
                while (nz) {
                    const int bit = __ffs((int)nz) - 1;  // 8*i + 7
                    atomicAdd(&lhist[(word >> (bit - 7)) & 255u], 1u);
                    nz &= nz - 1;
                }
                st[pxl * RSW + ktl * 8 + 4 * half + g] = word;
            }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) zero_count += __shfl_xor(zero_count, o, 64);
            if (lane == 0 && zero_count) atomicAdd(&lhist[zero_sym], zero_count);
        }
        __syncthreads();

        // ---- symbols leave as rows of ktg*32 bytes per pixel ----
        const int kbase = kt0 * 32;
        const int row_words = ktg * 8;
        for (int idx = tid; idx < PT * row_words; idx += kWideThreads) {
            const int row = idx / row_words, col = idx - row * row_words;
            const int64_t px = px0 + row;
            const int k = kbase + 4 * col;
            if (px < p.P && k < C) {
                const uint32_t word = st[row * RSW + col];
                uint8_t* dst = p.syms + px * C + k;
                if constexpr (VEC) {
                    *reinterpret_cast<uint32_t*>(dst) = word;
                } else {
                    for (int i = 0; i < 4 && k + i < C; i++) dst[i] = (uint8_t)(word >> (8 * i));
                }
            }
        }
    }
    __syncthreads();
    // one row of partial counts per workgroup: nothing to clear beforehand, no global atomics
    const int K = 1 << p.bits;
    if (tid < K) p.hist_parts[(size_t)(blockIdx.x + blockIdx.y * gridDim.x) * K + tid] = lhist[tid];
}

static hipError_t launch_wide(const BasisDevice& b, const float* d_x, int64_t P, int64_t HW, int layout, float delta,
                              int bits, uint8_t* d_syms, const CoderScratch& cs, int* n_parts, hipStream_t s) {
    WideParams p{};
    p.x = d_x;
    p.basis16 = b.fwd16;
    p.mu = b.mu;
    p.Trow = b.T;
    p.P = P;
    p.HW = HW;
    p.C = b.C;
    p.ncs = b.Cpad / 32;
    p.bits = bits;
    p.inv_delta = (float)(1.0 / (double)delta);
    p.delta = delta;
    // see launch_rows for the bound behind these two
    p.kappa = 1.9073486e-6f /* 2^-19 */ * b.row_norm * p.inv_delta;
    p.tau_min = 4.7683716e-7f /* 2^-21 */ * (float)(1 << (bits - 1));
    p.syms = d_syms;
    p.hist_parts = cs.hist_parts;
    p.ctrl = cs.ctrl;
    p.lookback = cs.lookback;
    p.n_groups = cs.n_groups;
    if (!p.x || !p.basis16 || !p.mu || !p.Trow || !p.syms || !p.hist_parts || !p.ctrl || !p.lookback)
        return hipErrorInvalidValue;  // (a field left out would be a wild pointer on the device)
    const int ncs = p.ncs;
    // Pixel tile: the larger it is the fewer times the basis streams through; the tile (both f16 parts) and the
    // staging rows have to fit LDS, and a small tensor is better off with more, smaller workgroups.
    const size_t lds_cap = 150 * 1024;
    int PT = 0, ktg = 0, kgroups = 1;
    int64_t px_tiles = 0;
    size_t lds = 0;
    for (int cand = 128; cand >= 32; cand /= 2) {
        px_tiles = (P + cand - 1) / cand;
        // split the coefficient range over workgroup rows only when the pixel tiles alone leave the chip idle
        kgroups = (int)((256 + px_tiles - 1) / px_tiles);
        if (kgroups < 1) kgroups = 1;
        ktg = (ncs + kgroups - 1) / kgroups;
        if (ktg > 16) ktg = 16;  // bounds the staging rows
        if (ktg > ncs) ktg = ncs;
        kgroups = (ncs + ktg - 1) / ktg;
        lds = (size_t)cand * (b.Cpad + 8) * 4 + sizeof(uint32_t) * (size_t)cand * (ktg * 8 + 1);
        PT = cand;
        if (lds <= lds_cap && (px_tiles >= 256 || cand == 32)) break;
    }
    if (lds > 158 * 1024) return hipErrorInvalidValue;  // not reachable for C <= 1024
    p.kt_per_group = ktg;
    p.px_tiles = px_tiles;
    int64_t gx = px_tiles;
    if (gx * kgroups > kMaxHistParts) gx = kMaxHistParts / kgroups;
    dim3 grid((unsigned)gx, (unsigned)kgroups);
    *n_parts = (int)(gx * kgroups);
    const bool vec = (b.C % 4) == 0;
    hipError_t el = hipSuccess;
#define FMTC_WIDE(PTV, LAY, VEC)                                                                                 \
    do {                                                                                                         \
        hipError_t ea = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_project_quantize_wide<PTV, LAY, VEC>), \
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);              \
        if (ea != hipSuccess) return ea;                                                                         \
        el = launch(K_PROJECT, k_project_quantize_wide<PTV, LAY, VEC>, grid, dim3(kWideThreads), lds, s, p);     \
    } while (0)
#define FMTC_WIDE_PT(LAY, VEC)                                                                                   \
    do {                                                                                                         \
        if (PT == 128) FMTC_WIDE(128, LAY, VEC);                                                                 \
        else if (PT == 64) FMTC_WIDE(64, LAY, VEC);                                                              \
        else FMTC_WIDE(32, LAY, VEC);                                                                            \
    } while (0)
    if (layout == FMTC_NHWC) { if (vec) FMTC_WIDE_PT(FMTC_NHWC, true); else FMTC_WIDE_PT(FMTC_NHWC, false); }
    else                     { if (vec) FMTC_WIDE_PT(FMTC_NCHW, true); else FMTC_WIDE_PT(FMTC_NCHW, false); }
#undef FMTC_WIDE_PT
#undef FMTC_WIDE
    return el;
}

// ---------------------------------------------------------------------------
// Narrow tensors (at most 160 channels after padding to 32).  One wavefront owns 32 pixels
// for all coefficients.  The contraction runs on the f16 matrix cores with every fp32 operand
// split in two f16 parts, v = hi + lo / 2^11 (hi = v rounded to f16, lo = 2^11 times the rest
// rounded to f16: 22 significant bits in all, and the scaling keeps lo out of the subnormals):
//   y = sum T_hi x_hi  +  2^-11 (sum T_hi x_lo + sum T_lo x_hi)
// with exact products and fp32 accumulation (v_mfma_f32_32x32x16_f16, three instructions per
// 16 channels where the fp32 instruction needs eight four times as long).  Measured against
// fp64 the result is as close as the fp32 instruction's; what is left of the error is bounded
// per pixel by a multiple of |x - mu|_2 and handled by the exact decision below.
// Lane (pixel r, half h) loads its pixel's channels 16j + 8h .. 16j + 8h + 7, j = 0 .. Cpad/16 - 1,
// straight from global memory into registers (the contraction index may be walked in any order
// as long as both operands agree, so no transpose through LDS is needed); the next tile's loads
// are issued as soon as this tile's values are converted.  The basis sits in LDS in operand
// order (see pack_operand16 on the host), rows of a tile permuted so that a lane ends up with
// 16 consecutive coefficients of its pixel: one 16-byte store of symbols per tile.  The
// quantizer of tile kt is scheduled between the matrix instructions of tile kt+1.
// Histogram: interleaved LDS copies per wavefront.
// ---------------------------------------------------------------------------
// Bit pattern of u clamped between the patterns of lo and hi (positive floats: their order is the order of their
// patterns as signed integers).  Compared as integers so that every input ends in range: a negative u (sign bit set)
// below lo, a NaN at one end or the other -- the result indexes the histogram.
__device__ __forceinline__ uint32_t clamp_pattern(float u, float lo, float hi) {
    const int ui = __builtin_bit_cast(int, u), li = __builtin_bit_cast(int, lo), hi_i = __builtin_bit_cast(int, hi);
    const int c = ui < li ? li : (ui > hi_i ? hi_i : ui);
    return (uint32_t)c;
}

constexpr int kHistLanes = 16;  // histogram copies per wavefront in the narrow-tensor kernel
constexpr int kFixList = 64;    // values per wavefront waiting for their exact decision

// LDS traffic of one wavefront completes in order; this keeps the compiler from moving it across the point
__device__ __forceinline__ void wave_sync_lds() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

struct RowParams {
    const float* x;
    const uint16_t* basis16;  // fwd16 packing
    const float* mu;          // [Cpad]
    const float* Trow;        // [C][C] row major, for the exact decisions
    int64_t P, HW;
    int C, bits;
    int active_tiles;         // 32-coefficient tiles up to the basis' last row that is not all zero
    float inv_delta, delta;
    float kappa;              // distance to a rounding boundary (in steps) below which a value of a pixel with
                              // |x - mu|_2 = 1 is decided exactly
    float tau_min;            // floor of that distance
    int64_t n_tiles;          // 32-pixel tiles
    uint8_t* syms;
    uint32_t* hist_parts;
    CoderCtrl* ctrl;
    unsigned long long* lookback;
    uint32_t n_groups;
    PackParams pk;            // FUSED only: where the container goes
};

// FUSED: the same projection and quantizer, but the symbols of a chunk stay in LDS and the wavefront packs them
// with a code table fixed beforehand (no histogram, nothing but the container leaves the kernel).  Needs
// C = 32 NCT in {32, 64, 128} and chunks of 4096 symbols, i.e. 4 / NCT whole pixel tiles; the grid must not exceed
// what the device holds at once (a chunk's position in the payload comes from the workgroups before it), and the
// look-back words and the control block must be clear when the kernel starts.
// WAVES wavefronts per workgroup (4, or 8 sharing one copy of a large basis); the register budget is set so that
// rows_waves_per_simd() wavefronts fit a SIMD: a wavefront spends most of a tile's time waiting for its pixels,
// and the second (third, fourth) one's arithmetic fills that time.
constexpr int rows_waves_per_simd(int nct, bool fused, int waves) {
    return fused ? 1 : (waves == 8 ? 2 : (nct == 1 ? 4 : (nct <= 3 ? 2 : 1)));
}
template <int NCT, int LAYOUT, bool VEC, bool FUSED = false, int WAVES = 4, int WPS = rows_waves_per_simd(NCT, FUSED, WAVES)>
__global__ __launch_bounds__(WAVES * 64) __attribute__((amdgpu_waves_per_eu(WPS, WPS)))
void k_project_quantize_rows(RowParams p) {
    constexpr int THREADS = WAVES * 64;
    static_assert(WAVES == 4 || (WAVES == 8 && !FUSED), "workgroup shape");
    // SEQ: contraction, then quantizer, tile by tile with one pair of accumulators (see process_tile)
    constexpr bool SEQ = WPS >= 3 || WAVES == 8;
    constexpr int NJ = NCT * 2;  // steps of 16 channels
    extern __shared__ __align__(16) uint4 basis16[];  // [NCT][NJ][2][64], then the histograms
    __shared__ __align__(16) float s_mu[NCT * 32];
    __shared__ uint32_t s_fix_list[WAVES][kFixList];
    __shared__ uint32_t s_fix_tile[WAVES][kFixList];
    __shared__ uint32_t s_fix_count[WAVES];
    __shared__ uint32_t s_red[WAVES * 256];  // per (wavefront, bin) sums of the histogram copies
    // Histogram: kHistLanes interleaved copies per wavefront (bin s of copy q at word s * kHistLanes + q), lane l
    // counts in copy l % kHistLanes.  Most symbols of a tile are the same few values: with one copy the LDS
    // would serialise up to 64 additions to one word per instruction, and the reads of the basis queue up
    // behind them.
    const int K = 1 << p.bits;
    uint32_t* whist = reinterpret_cast<uint32_t*>(basis16 + NCT * NJ * 2 * 64);  // [WAVES][K * kHistLanes]
    // FUSED: in place of the histograms, the four wavefronts' chunks of symbols (4096 bytes each, stream order)
    // and the packer's tables and images
    constexpr int TPC = FUSED ? 4 / NCT : 1;  // pixel tiles per chunk
    uint8_t* sym_tiles = reinterpret_cast<uint8_t*>(whist);
    PackShared& S = *reinterpret_cast<PackShared*>(sym_tiles + 4 * 4096);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wavefront-uniform by construction
    const int half = lane >> 5, l32 = lane & 31;
    const int C = p.C;
    // this lane's half of its pixel as loaded: xr[8j + e] = x[px][16j + 8h + e]
    float xr[NJ * 8];
    auto load_pixels = [&](int64_t tile) {
        const int64_t px = tile * 32 + l32;
        const bool px_ok = px < p.P;
        if constexpr (LAYOUT == FMTC_NHWC && VEC) {
            if (C == NCT * 32 && tile * 32 + 32 <= p.P) {  // wavefront-uniform: nothing to mask, nothing to fill
                const float4* row = reinterpret_cast<const float4*>(p.x + px * (NCT * 32)) + 2 * half;
#pragma unroll
                for (int j = 0; j < NJ; j++)
#pragma unroll
                    for (int q = 0; q < 2; q++) {
                        const float4 v = row[4 * j + q];
                        xr[8 * j + 4 * q] = v.x; xr[8 * j + 4 * q + 1] = v.y;
                        xr[8 * j + 4 * q + 2] = v.z; xr[8 * j + 4 * q + 3] = v.w;
                    }
                return;
            }
            const float4* row = reinterpret_cast<const float4*>(p.x + (px_ok ? px : 0) * C) + 2 * half;
#pragma unroll
            for (int j = 0; j < NJ; j++)
#pragma unroll
                for (int q = 0; q < 2; q++) {
                    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (px_ok && 16 * j + 8 * half + 4 * q < C) v = row[4 * j + q];
                    xr[8 * j + 4 * q] = v.x; xr[8 * j + 4 * q + 1] = v.y;
                    xr[8 * j + 4 * q + 2] = v.z; xr[8 * j + 4 * q + 3] = v.w;
                }
        } else {
            int64_t base = 0, stride = 1;
            if constexpr (LAYOUT == FMTC_NHWC) {
                base = (px_ok ? px : 0) * C;
            } else {
                const int64_t pp = px_ok ? px : 0;
                const int64_t n = pp / p.HW;
                base = n * (int64_t)C * p.HW + (pp - n * p.HW);
                stride = p.HW;
            }
#pragma unroll
            for (int j = 0; j < NJ; j++)
#pragma unroll
                for (int e = 0; e < 8; e++) {
                    const int c = 16 * j + 8 * half + e;
                    xr[8 * j + e] = (px_ok && c < C) ? p.x[base + (int64_t)c * stride] : 0.f;
                }
        }
    };
    // the first tile's pixels come from HBM: their loads go out before anything else
    int64_t tile = ((int64_t)blockIdx.x * WAVES + wave) * TPC;
    if (tile < p.n_tiles) load_pixels(tile);
    if constexpr (!FUSED) zero_coder_scratch(p.ctrl, p.lookback, p.n_groups);

    // the basis goes from global memory straight into LDS, 16 bytes per lane and instruction
    {
        const uint4* src = reinterpret_cast<const uint4*>(p.basis16);
#pragma unroll
        for (int i = 0; i < (NCT * NCT * 256 + THREADS - 1) / THREADS; i++)
            if (THREADS * i + 64 * wave < NCT * NCT * 256)  // whole wavefronts
                __builtin_amdgcn_global_load_lds(src + tid + THREADS * i, &basis16[THREADS * i + 64 * wave], 16, 0, 0);
    }
    if (tid < NCT * 32) s_mu[tid] = p.mu[tid];
    if constexpr (!FUSED) {
        for (int i = tid; i < WAVES * K * kHistLanes; i += THREADS) whist[i] = 0u;
    } else {
        S.tab[tid] = p.pk.enc_table[tid];
        if (tid == 0) {
            S.max_len = p.pk.static_max_len;
            S.payload_bits = 0ull;
        }
        if (blockIdx.x == 0) p.pk.stream[kHeaderBytes + tid] = (uint8_t)(p.pk.enc_table[tid] >> 56);  // the container's length table
        pack_clear_image(S, wave, lane);
    }

    const int zero_sym = 1 << (p.bits - 1);
    const float lo = (float)(-zero_sym), hi = (float)(zero_sym - 1), zero_f = (float)zero_sym;
    const float inv_delta = p.inv_delta;
    const float inv_delta_lo = p.inv_delta * (1.f / 2048.f);
    // Rounding, offset and conversion in one addition: for |t| < 2^22, t + (1.5 * 2^23 + 2^(b-1)) rounds (half to
    // even, the unit in the last place there being 1) to the number whose bit pattern is kMagicBits + 2^(b-1) +
    // rne(t); clamped between the patterns of symbol 0 and symbol 2^b - 1 its lowest byte is the symbol, and
    // subtracting the constant again gives rne(t) for the distance to the rounding boundary.  Larger |t| clamp the
    // same way (their distance is then meaningless and large: such a value is decided exactly, like any flagged one).
    constexpr uint32_t kMagicBits = 0x4B400000u;  // 1.5 * 2^23
    const float magic = 12582912.f + (float)zero_sym;
    const float magic_lo = 12582912.f, magic_hi = 12582912.f + (float)(2 * zero_sym - 1);
    uint32_t* wh0 = whist + wave * K * kHistLanes;          // this wavefront's histogram, copy 0
    uint32_t* wh = wh0 + (lane & (kHistLanes - 1));         // bin s of this lane's copy: wh[s * kHistLanes]
    // count of the symbol in the clamped pattern `ub` (kMagicBits + symbol): the LDS address is one shift-and-add
    // from the pattern itself (the constant is folded into the base; the arithmetic wraps)
    static_assert(kHistLanes * sizeof(uint32_t) == 64, "shift of the histogram address");
    typedef __attribute__((address_space(3))) uint32_t lds_u32;
    const uint32_t wh_magic = (uint32_t)(uintptr_t)(lds_u32*)wh - (kMagicBits << 6);
    auto hist_add = [&](uint32_t ub) {
        __hip_atomic_fetch_add((lds_u32*)(uintptr_t)((ub << 6) + wh_magic), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    };
    uint32_t* fix_list = s_fix_list[wave];
    uint32_t* fix_tile = s_fix_tile[wave];
    uint32_t* fix_count = &s_fix_count[wave];
    if (lane == 0) *fix_count = 0u;

    // the first tile's pixels are on their way while the basis lands; every wavefront of the workgroup takes
    // part in the barrier, with or without a tile
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wavefront's part of the basis has landed in LDS
    __syncthreads();

    int64_t chunk_px0 = 0;  // FUSED: first pixel of the chunk this wavefront is working on
    // ---- exact decision where the fast pass can not be trusted (rare) ----
    // A tile notes the values that lie too close to a rounding boundary in the wavefront's list: tile, pixel
    // lane, coefficient and the symbol already stored and counted.  When the list is full, and after the
    // wavefront's last tile, the listed values are recomputed in fp64 (same arithmetic as the definition: sum of
    // T[k][c] * (x[c] - mu[c]), divided by the step), four per round, all loads of a round in flight
    // together, and the stored symbol and the histogram are patched where the decision differs.
    auto resolve_list = [&]() {
        // the symbols that get patched were stored by other lanes of this wavefront: those stores are
        // acknowledged before the patches go out (this also waits for the next tile's loads; rare)
        __builtin_amdgcn_s_waitcnt(0x0F70);
        const uint32_t n = (uint32_t)__builtin_amdgcn_readfirstlane((int)*fix_count);
        for (uint32_t base = 0; base < n; base += 4) {
            const uint32_t idx = base + (uint32_t)(lane >> 4);
            const bool active = idx < n;
            const uint32_t e = active ? fix_list[idx] : 0u;
            const int k = (int)(e & 255u), pl = (int)((e >> 8) & 31u);
            const uint32_t old = e >> 13;
            const int64_t qpx = (int64_t)fix_tile[idx < (uint32_t)kFixList ? idx : 0] * 32 + pl;
            int64_t xbase, xstride;
            if constexpr (LAYOUT == FMTC_NHWC) {
                xbase = qpx * C;
                xstride = 1;
            } else {
                const int64_t n_img = qpx / p.HW;
                xbase = n_img * (int64_t)C * p.HW + (qpx - n_img * p.HW);
                xstride = p.HW;
            }
            float tv[2 * NCT], xv[2 * NCT], mv[2 * NCT];
#pragma unroll
            for (int it = 0; it < 2 * NCT; it++) {
                const int c = (lane & 15) + 16 * it;
                const bool in = active && c < C;
                tv[it] = in ? p.Trow[(size_t)k * C + c] : 0.f;
                xv[it] = in ? p.x[xbase + c * xstride] : 0.f;
                mv[it] = in ? s_mu[c] : 0.f;
            }
            double part = 0.0;
#pragma unroll
            for (int it = 0; it < 2 * NCT; it++) part += (double)tv[it] * ((double)xv[it] - (double)mv[it]);
#pragma unroll
            for (int o = 8; o > 0; o >>= 1) part += __shfl_xor(part, o, 64);  // stays inside the 16-lane group
            double qd = rint(part / (double)p.delta);
            qd = fmin(fmax(qd, (double)lo), (double)hi);
            const uint32_t sfix = (uint32_t)((int)qd + zero_sym);
            if (active && (lane & 15) == 0 && sfix != old) {
                if constexpr (FUSED) {
                    // the listed tiles are those of the chunk in this wavefront's LDS tile
                    sym_tiles[wave * 4096 + ((qpx - chunk_px0) * C + k)] = (uint8_t)sfix;
                } else {
                    atomicSub(&wh0[old * kHistLanes], 1u);
                    atomicAdd(&wh0[sfix * kHistLanes], 1u);
                    p.syms[qpx * C + k] = (uint8_t)sfix;
                }
            }
        }
        wave_sync_lds();
        if (lane == 0) *fix_count = 0u;
        wave_sync_lds();
    };
    auto process_tile = [&](const int64_t tile, const int64_t next_tile) {
        const int64_t px = tile * 32 + l32;
        const bool px_ok = px < p.P;
        // ---- mean removed, split into the two f16 parts (padding channels hold 0 - 0) ----
        halfx8 xh[NJ], xl[NJ];
        float n2 = 0.f;
        auto split = [&](bool clamp) {
            n2 = 0.f;
#pragma unroll
            for (int j = 0; j < NJ; j++)
#pragma unroll
                for (int q = 0; q < 2; q++) {
                    const float4 m = *reinterpret_cast<const float4*>(&s_mu[16 * j + 8 * half + 4 * q]);
                    const float mv[4] = {m.x, m.y, m.z, m.w};
#pragma unroll
                    for (int i = 0; i < 4; i++) {
                        float v = xr[8 * j + 4 * q + i] - mv[i];
                        n2 = __builtin_fmaf(v, v, n2);
                        if (clamp) v = __builtin_amdgcn_fmed3f(v, -60000.f, 60000.f);
                        const _Float16 vh = (_Float16)v;
                        xh[j][4 * q + i] = vh;
                        // 2^11 (v - vh), exact (one multiply-add that takes the f16 operand as it is)
                        xl[j][4 * q + i] = (_Float16)__builtin_fmaf((float)vh, -2048.f, v * 2048.f);
                    }
                }
        };
        split(false);
        n2 += __shfl_xor(n2, 32, 64);  // the other half of the pixel
        // a pixel too large for f16 (or not finite) is decided exactly, every coefficient of it; its values are
        // clamped on the way into the matrix cores so that what comes out stays finite
        const bool force = !(n2 < 1.0e9f);
        if (__builtin_expect(__any(force), 0)) split(true);
        const float tau = fminf(fmaxf(p.kappa * __builtin_sqrtf(n2), p.tau_min), 0.125f);
        const float near_limit = force ? -1.f : 0.5f - tau;
        // the raw registers are free: the next tile's loads are in flight during this tile's arithmetic.  (With
        // three or more wavefronts per SIMD the others' arithmetic covers the loads, and registers held by loads in
        // flight across the whole tile are what would not fit: there the loads go out after the tile.)
        if (WPS < 3 && next_tile < p.n_tiles) load_pixels(next_tile);

        auto project_tile = [&](int kt, floatx16& am, floatx16& ac) {
            if (kt >= p.active_tiles) {  // all rows of the tile are zero (truncated basis): so are its coefficients
#pragma unroll
                for (int r = 0; r < 16; r++) { am[r] = 0.f; ac[r] = 0.f; }
                return;
            }
            // (the first step starts from the instruction's constant zero: no registers to clear)
            const floatx16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < NJ; j++) {
                const uint4 th4 = basis16[((kt * NJ + j) * 2) * 64 + lane];
                const uint4 tl4 = basis16[((kt * NJ + j) * 2 + 1) * 64 + lane];
                const halfx8 th = __builtin_bit_cast(halfx8, th4), tl = __builtin_bit_cast(halfx8, tl4);
                am = __builtin_amdgcn_mfma_f32_32x32x16_f16(th, xh[j], j ? am : zero, 0, 0, 0);
                ac = __builtin_amdgcn_mfma_f32_32x32x16_f16(th, xl[j], j ? ac : zero, 0, 0, 0);
                ac = __builtin_amdgcn_mfma_f32_32x32x16_f16(tl, xh[j], ac, 0, 0, 0);
            }
        };
        // accumulator r = 4g + i of lane (pixel, h) is coefficient kt*32 + 16h + 4g + i of the pixel.
        // Quantizer, histogram and store of one tile with ragged edges (pixels past P, coefficients past C).
        auto quantize_tile = [&](const floatx16& am, const floatx16& ac, int kt, uint32_t (&word)[4]) -> float {
            const int k0 = kt * 32 + 16 * half;
            float maxd = 0.f;
#pragma unroll
            for (int g = 0; g < 4; g++) {
                word[g] = 0u;
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    const float t = __builtin_fmaf(ac[4 * g + i], inv_delta_lo, am[4 * g + i] * inv_delta);
                    const float q = __builtin_rintf(t);  // round half to even
                    maxd = fmaxf(maxd, fabsf(t - q));
                    const float qc = __builtin_amdgcn_fmed3f(q, lo, hi) + zero_f;  // clamped level, as a symbol
                    word[g] = __builtin_amdgcn_cvt_pk_u8_f32(qc, i, word[g]);
                }
            }
            if (px_ok) {
#pragma unroll
                for (int r = 0; r < 16; r++)
                    if (k0 + r < C) {
                        const uint32_t sy = (word[r >> 2] >> (8 * (r & 3))) & 255u;
                        if constexpr (FUSED) {
                            sym_tiles[wave * 4096 + ((px - chunk_px0) * C + k0 + r)] = (uint8_t)sy;
                        } else {
                            atomicAdd(&wh[sy * kHistLanes], 1u);
                            p.syms[px * C + k0 + r] = (uint8_t)sy;
                        }
                    }
            }
            return maxd;
        };
        auto note_tile = [&](const floatx16& am, const floatx16& ac, int kt, const uint32_t (&word)[4]) {
            const int k0 = kt * 32 + 16 * half;
            uint32_t near_mask = 0;
#pragma unroll
            for (int r = 0; r < 16; r++) {
                const float t = __builtin_fmaf(ac[r], inv_delta_lo, am[r] * inv_delta);
                if (!(fabsf(t - __builtin_rintf(t)) <= near_limit) && px_ok && k0 + r < C) near_mask |= 1u << r;
            }
            // at most 64 * 16 new entries would not fit: resolve what is there first if this tile could overflow
            const uint32_t incoming = wave_sum((uint32_t)__popc(near_mask));
            if (*fix_count + incoming > (uint32_t)kFixList) resolve_list();
            if (incoming > (uint32_t)kFixList) {
                // more flagged values than the list holds (a step so fine that the fast pass decides almost
                // nothing, or pixels out of its range): 16 passes, one accumulator each, at most 64 entries per pass
#pragma unroll 1
                for (int r = 0; r < 16; r++) {
                    if ((near_mask >> r) & 1u) {
                        const uint32_t slot = atomicAdd(fix_count, 1u);
                        fix_list[slot] = (uint32_t)(k0 + r) | ((uint32_t)l32 << 8) |
                                         (((word[r >> 2] >> (8 * (r & 3))) & 255u) << 13);
                        fix_tile[slot] = (uint32_t)tile;
                    }
                    wave_sync_lds();
                    resolve_list();
                }
            } else {
                while (near_mask) {
                    const int r = __ffs((int)near_mask) - 1;
                    near_mask &= near_mask - 1;
                    uint32_t sy = 0;
#pragma unroll
                    for (int g = 0; g < 4; g++)
                        if (g == (r >> 2)) sy = (word[g] >> (8 * (r & 3))) & 255u;
                    const uint32_t slot = atomicAdd(fix_count, 1u);
                    fix_list[slot] = (uint32_t)(k0 + r) | ((uint32_t)l32 << 8) | (sy << 13);
                    fix_tile[slot] = (uint32_t)tile;
                }
                wave_sync_lds();
            }
        };

        // whole pixel tile, and every lane's 16 coefficients of a tile all inside C or all outside (wavefront-uniform)
        const bool full = (tile * 32 + 32 <= p.P) && (C % 16 == 0);
        floatx16 am, ac;
        project_tile(0, am, ac);
        if (full && SEQ) {
            // Several wavefronts per SIMD: the others fill the shadow of this one's matrix instructions, and one
            // pair of accumulators (not two) is what lets them fit: contraction, then quantizer, tile by tile.
#pragma unroll
            for (int kt = 0; kt < NCT; kt++) {
                if (kt) project_tile(kt, am, ac);
                uint32_t word[4] = {0u, 0u, 0u, 0u};
                float maxd = 0.f;
                const bool k_ok = kt * 32 + 16 * half < C;  // false only in the upper half of a padded last tile
                uint32_t ub[16];
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    const float t = __builtin_fmaf(ac[r], inv_delta_lo, am[r] * inv_delta);
                    const float u = t + magic;  // round half to even
                    maxd = fmaxf(maxd, fabsf(t - (u - magic)));
                    ub[r] = clamp_pattern(u, magic_lo, magic_hi);
                    if constexpr (!FUSED)
                        if (k_ok) hist_add(ub[r]);
                }
#pragma unroll
                for (int g = 0; g < 4; g++)
                    word[g] = __builtin_amdgcn_perm(__builtin_amdgcn_perm(ub[4 * g + 3], ub[4 * g + 2], 0x0c0c0400u),
                                                    __builtin_amdgcn_perm(ub[4 * g + 1], ub[4 * g], 0x0c0c0400u), 0x05040100u);
                if constexpr (FUSED) {
                    *reinterpret_cast<uint4*>(sym_tiles + wave * 4096 + ((px - chunk_px0) * C + kt * 32 + 16 * half)) =
                        make_uint4(word[0], word[1], word[2], word[3]);
                } else if (k_ok) {
                    *reinterpret_cast<uint4*>(p.syms + px * C + kt * 32 + 16 * half) =
                        make_uint4(word[0], word[1], word[2], word[3]);
                }
                if (__builtin_expect(__any(!(maxd <= near_limit) && k_ok), 0)) note_tile(am, ac, kt, word);
            }
        } else if (full) {
            // One wavefront per SIMD: nothing else fills the shadow of the matrix pipe, so the quantizer of tile
            // kt is issued between the matrix instructions of tile kt + 1 -- after each step of the contraction
            // the share of the previous tile's 16 values that keeps both in step.
#pragma unroll
            for (int kt = 0; kt < NCT; kt++) {
                floatx16 nm, nc;
#pragma unroll
                for (int r = 0; r < 16; r++) { nm[r] = 0.f; nc[r] = 0.f; }
                uint32_t word[4] = {0u, 0u, 0u, 0u};
                uint32_t ub[16];
                float maxd = 0.f;
                const bool k_ok = kt * 32 + 16 * half < C;  // false only in the upper half of a padded last tile
                auto quantize_value = [&](int r) {
                    const float t = __builtin_fmaf(ac[r], inv_delta_lo, am[r] * inv_delta);
                    const float u = t + magic;  // round half to even
                    maxd = fmaxf(maxd, fabsf(t - (u - magic)));
                    ub[r] = clamp_pattern(u, magic_lo, magic_hi);
                    if constexpr (!FUSED)
                        if (k_ok) hist_add(ub[r]);
                    if ((r & 3) == 3)
                        word[r >> 2] = __builtin_amdgcn_perm(__builtin_amdgcn_perm(ub[r], ub[r - 1], 0x0c0c0400u),
                                                             __builtin_amdgcn_perm(ub[r - 2], ub[r - 3], 0x0c0c0400u), 0x05040100u);
                };
                if (kt + 1 < NCT) {
#pragma unroll
                    for (int j = 0; j < NJ; j++) {
                        const uint4 th4 = basis16[(((kt + 1) * NJ + j) * 2) * 64 + lane];
                        const uint4 tl4 = basis16[(((kt + 1) * NJ + j) * 2 + 1) * 64 + lane];
                        const halfx8 th = __builtin_bit_cast(halfx8, th4), tl = __builtin_bit_cast(halfx8, tl4);
                        nm = __builtin_amdgcn_mfma_f32_32x32x16_f16(th, xh[j], nm, 0, 0, 0);
                        nc = __builtin_amdgcn_mfma_f32_32x32x16_f16(th, xl[j], nc, 0, 0, 0);
                        nc = __builtin_amdgcn_mfma_f32_32x32x16_f16(tl, xh[j], nc, 0, 0, 0);
#pragma unroll
                        for (int r = 16 * j / NJ; r < 16 * (j + 1) / NJ; r++) quantize_value(r);
                    }
                } else {
#pragma unroll
                    for (int r = 0; r < 16; r++) quantize_value(r);
                }
                // C is a multiple of 16: every lane's 16 symbols are a 16-byte aligned piece of its pixel's row
                if constexpr (FUSED) {
                    *reinterpret_cast<uint4*>(sym_tiles + wave * 4096 + ((px - chunk_px0) * C + kt * 32 + 16 * half)) =
                        make_uint4(word[0], word[1], word[2], word[3]);
                } else if (k_ok) {
                    *reinterpret_cast<uint4*>(p.syms + px * C + kt * 32 + 16 * half) =
                        make_uint4(word[0], word[1], word[2], word[3]);
                }
                if (__builtin_expect(__any(!(maxd <= near_limit) && k_ok), 0)) note_tile(am, ac, kt, word);
                am = nm;
                ac = nc;
            }
        } else if (SEQ) {
#pragma unroll
            for (int kt = 0; kt < NCT; kt++) {
                uint32_t word[4];
                if (kt) project_tile(kt, am, ac);
                const float maxd = quantize_tile(am, ac, kt, word);
                if (__builtin_expect(__any(!(maxd <= near_limit) && px_ok), 0)) note_tile(am, ac, kt, word);
            }
        } else {
#pragma unroll
            for (int kt = 0; kt < NCT; kt++) {
                floatx16 nm, nc;
                uint32_t word[4];
                if (kt + 1 < NCT) project_tile(kt + 1, nm, nc);
                const float maxd = quantize_tile(am, ac, kt, word);
                if (__builtin_expect(__any(!(maxd <= near_limit) && px_ok), 0)) note_tile(am, ac, kt, word);
                if (kt + 1 < NCT) { am = nm; ac = nc; }
            }
        }
    };
    if constexpr (FUSED) {
        // Chunk group g = the chunks 4g .. 4g + 3, one per wavefront; the workgroup takes groups blockIdx.x,
        // blockIdx.x + gridDim.x, ... in turn, so every group before one in progress is finished or in progress too.
        for (uint32_t group = blockIdx.x; group < p.pk.n_groups; group += gridDim.x) {
            const uint32_t ch = group * 4 + (uint32_t)wave;
            const int64_t tile0 = (int64_t)ch * TPC;
            const int64_t next_chunk_tile = ((int64_t)(group + gridDim.x) * 4 + wave) * TPC;  // past the end: no loads
            chunk_px0 = tile0 * 32;
            uint32_t clen = 0;
            if (ch < p.pk.n_chunks) {
                const uint64_t c0 = (uint64_t)ch * 4096u;
                clen = (uint32_t)((p.pk.V - c0 < 4096u) ? (p.pk.V - c0) : 4096u);
#pragma unroll
                for (int t = 0; t < TPC; t++) {
                    const int64_t tl = tile0 + t;
                    if (tl < p.n_tiles)  // wavefront-uniform
                        process_tile(tl, (t + 1 < TPC && tl + 1 < p.n_tiles) ? tl + 1
                                         : (group + gridDim.x < p.pk.n_groups ? next_chunk_tile : p.n_tiles));
                }
                if (*fix_count) resolve_list();
            }
            wave_sync_lds();  // the symbols other lanes wrote precede the reads below
            // register q of lane l: symbols 256q + 4l .. + 3 of the chunk (C is a multiple of 32: clen one of 4)
            uint32_t w[16];
#pragma unroll
            for (int q = 0; q < 16; q++) {
                const uint32_t o = 256u * q + 4u * (uint32_t)lane;
                w[q] = (o + 4u <= clen) ? *reinterpret_cast<const uint32_t*>(sym_tiles + wave * 4096 + o) : 0u;
            }
            pack_group<kPackStatic>(S, p.pk, group, w, clen, []() {});
        }
        return;
    } else {
        for (; tile < p.n_tiles; tile += (int64_t)gridDim.x * WAVES) {
            const int64_t next_tile = tile + (int64_t)gridDim.x * WAVES;
            process_tile(tile, next_tile);
            if (WPS >= 3 && next_tile < p.n_tiles) load_pixels(next_tile);
        }
    }
    if (*fix_count) resolve_list();
    __syncthreads();
    // One row of partial counts per workgroup: nothing to clear beforehand, no global atomics.  Every thread sums
    // the 16 copies of some (wavefront, bin) rows with 16-byte reads (a row is contiguous; reading one copy of
    // many bins instead would put all lanes on two banks), then the first K threads add the wavefronts.
    for (int row = tid; row < WAVES * K; row += THREADS) {
        const uint4* r4 = reinterpret_cast<const uint4*>(whist + (size_t)row * kHistLanes);
        uint32_t total = 0;
#pragma unroll
        for (int q = 0; q < kHistLanes / 4; q++) {
            const uint4 v = r4[q];
            total += (v.x + v.y) + (v.z + v.w);
        }
        s_red[row] = total;
    }
    __syncthreads();
    if (tid < K) {
        uint32_t total = 0;
#pragma unroll
        for (int q = 0; q < WAVES; q++) total += s_red[q * K + tid];
        p.hist_parts[(size_t)blockIdx.x * K + tid] = total;
    }
}

// ---------------------------------------------------------------------------
// 128 to 160 channels, channels last, a multiple of 16 of them: the same projection with the loops the other way
// round.  k_project_quantize_rows holds a whole pixel tile twice (the fp32 values of the next tile on their way in, the
// two f16 parts of this one) and one or two pairs of accumulators: 350 to 450 registers at four and five coefficient
// tiles, one wavefront per SIMD -- where a vector instruction issues every 8 clocks instead of every 4 and nothing
// covers a wait.  Here the channel steps are the outer loop: a step's eight channels per lane are converted when
// their turn comes and go into the accumulators of ALL coefficient tiles at once (32 NCT accumulator registers), and
// the pixels stream in through two small buffers of two steps each, across tile boundaries, so that between one and
// two buffers (4 to 8 KB per wavefront) are in flight at any time.  130 registers less at four tiles: two wavefronts
// per SIMD (eight on one copy of the basis) without spills.  A pixel too large for f16 needs no clamp here: what its
// infinities make of the matrix product stays in its own column of outputs, all of which are decided exactly, and
// the clamp of the quantizer keeps the histogram index in range whatever the value.
// ---------------------------------------------------------------------------
// NJA: the tensor's channel count / 16 (the launcher checks it), 2 NCT - 1 or 2 NCT.
template <int NCT, int WAVES, int NJA>
__global__ __launch_bounds__(WAVES * 64) __attribute__((amdgpu_waves_per_eu(WAVES / 4, WAVES / 4)))
void k_project_quantize_stream(RowParams p) {
    constexpr int THREADS = WAVES * 64;
    constexpr int NJ = NCT * 2;        // steps of 16 channels in the basis operand (of which the first NJA hold channels)
    static_assert(NJA == NJ || NJA == NJ - 1, "channel count");
    constexpr int NP = (NJ + 1) / 2;   // pairs of steps: the unit of the pixel buffers
    extern __shared__ __align__(16) uint4 basis16[];  // [NCT][NJ][2][64], then the histograms
    __shared__ __align__(16) float s_mu[NCT * 32];
    __shared__ uint32_t s_fix_list[WAVES][kFixList];
    __shared__ uint32_t s_fix_tile[WAVES][kFixList];
    __shared__ uint32_t s_fix_count[WAVES];
    __shared__ uint32_t s_red[WAVES * 256];
    const int K = 1 << p.bits;
    uint32_t* whist = reinterpret_cast<uint32_t*>(basis16 + NCT * NJ * 2 * 64);  // [WAVES][K * kHistLanes]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, l32 = lane & 31;
    constexpr int C = 16 * NJA;
    typedef float f4_t __attribute__((ext_vector_type(4)));

    // this lane's channels [16 j + 8 half, + 8) of its pixel, steps 2 pr and 2 pr + 1, of pixel tile `tile`
    auto load_pair = [&](int64_t tile, int pr, f4_t (&buf)[2][2]) __attribute__((always_inline)) {
        int64_t px = tile * 32 + l32;
        px = px < p.P ? px : p.P - 1;  // rows past the tensor repeat its last pixel; never stored or counted
        const f4_t* row = reinterpret_cast<const f4_t*>(p.x + px * C) + 2 * half;
#pragma unroll
        for (int u = 0; u < 2; u++) {
            const int j = 2 * pr + u;
            if (j < NJ && j < NJA) {  // wavefront-uniform
                buf[u][0] = row[4 * j];
                buf[u][1] = row[4 * j + 1];
            }
        }
    };
    const int64_t stride = (int64_t)gridDim.x * WAVES;
    int64_t tile = (int64_t)blockIdx.x * WAVES + wave;
    f4_t bufA[2][2], bufB[2][2];
    if (tile < p.n_tiles) {
        load_pair(tile, 0, bufA);
        if (NP > 1) load_pair(tile, 1, bufB);
    }
    zero_coder_scratch(p.ctrl, p.lookback, p.n_groups);
    {
        const uint4* src = reinterpret_cast<const uint4*>(p.basis16);
#pragma unroll
        for (int i = 0; i < (NCT * NCT * 256 + THREADS - 1) / THREADS; i++)
            if (THREADS * i + 64 * wave < NCT * NCT * 256)  // whole wavefronts
                __builtin_amdgcn_global_load_lds(src + tid + THREADS * i, &basis16[THREADS * i + 64 * wave], 16, 0, 0);
    }
    if (tid < NCT * 32) s_mu[tid] = p.mu[tid];
    for (int i = tid; i < WAVES * K * kHistLanes; i += THREADS) whist[i] = 0u;

    const int zero_sym = 1 << (p.bits - 1);
    const float lo = (float)(-zero_sym), hi = (float)(zero_sym - 1);
    const float inv_delta = p.inv_delta;
    const float inv_delta_lo = p.inv_delta * (1.f / 2048.f);
    constexpr uint32_t kMagicBits = 0x4B400000u;  // 1.5 * 2^23: see k_project_quantize_rows
    const float magic = 12582912.f + (float)zero_sym;
    const float magic_lo = 12582912.f, magic_hi = 12582912.f + (float)(2 * zero_sym - 1);
    uint32_t* wh0 = whist + wave * K * kHistLanes;
    uint32_t* wh = wh0 + (lane & (kHistLanes - 1));
    static_assert(kHistLanes * sizeof(uint32_t) == 64, "shift of the histogram address");
    typedef __attribute__((address_space(3))) uint32_t lds_u32;
    const uint32_t wh_magic = (uint32_t)(uintptr_t)(lds_u32*)wh - (kMagicBits << 6);
    auto hist_add = [&](uint32_t ub) {
        __hip_atomic_fetch_add((lds_u32*)(uintptr_t)((ub << 6) + wh_magic), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    };
    uint32_t* fix_list = s_fix_list[wave];
    uint32_t* fix_tile = s_fix_tile[wave];
    uint32_t* fix_count = &s_fix_count[wave];
    if (lane == 0) *fix_count = 0u;
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wavefront's part of the basis has landed in LDS
    __syncthreads();

    // exact decision of the listed values (as in k_project_quantize_rows)
    auto resolve_list = [&]() __attribute__((always_inline)) {
        __builtin_amdgcn_s_waitcnt(0x0F70);
        const uint32_t n = (uint32_t)__builtin_amdgcn_readfirstlane((int)*fix_count);
        for (uint32_t base = 0; base < n; base += 4) {
            const uint32_t idx = base + (uint32_t)(lane >> 4);
            const bool active = idx < n;
            const uint32_t e = active ? fix_list[idx] : 0u;
            const int k = (int)(e & 255u), pl = (int)((e >> 8) & 31u);
            const uint32_t old = e >> 13;
            const int64_t qpx = (int64_t)fix_tile[idx < (uint32_t)kFixList ? idx : 0] * 32 + pl;
            double part = 0.0;
            if (active)
#pragma unroll 5
                for (int c = lane & 15; c < C; c += 16)
                    part += (double)p.Trow[(size_t)k * C + c] * ((double)p.x[qpx * C + c] - (double)s_mu[c]);
#pragma unroll
            for (int o = 8; o > 0; o >>= 1) part += __shfl_xor(part, o, 64);  // stays inside the 16-lane group
            double qd = rint(part / (double)p.delta);
            qd = fmin(fmax(qd, (double)lo), (double)hi);
            const uint32_t sfix = (uint32_t)((int)qd + zero_sym);
            if (active && (lane & 15) == 0 && sfix != old) {
                atomicSub(&wh0[old * kHistLanes], 1u);
                atomicAdd(&wh0[sfix * kHistLanes], 1u);
                p.syms[qpx * C + k] = (uint8_t)sfix;
            }
        }
        wave_sync_lds();
        if (lane == 0) *fix_count = 0u;
        wave_sync_lds();
    };

    // One pixel tile.  SWAP (a compile-time flag): the roles of the two buffers are exchanged (see the loop below).
    auto tile_body = [&](auto swap_c, const int64_t tile) __attribute__((always_inline)) {
        constexpr bool SWAP = decltype(swap_c)::value;
        const int64_t next_tile = tile + stride;
        const int64_t px = tile * 32 + l32;
        const bool px_ok = px < p.P;
        floatx16 am[NCT], ac[NCT];
        float n2 = 0.f;
        const floatx16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        // one step: this lane's eight channels converted, then into every coefficient tile's accumulators
        auto step = [&](int j, const f4_t (&raw)[2]) __attribute__((always_inline)) {
            halfx8 xh, xl;
#pragma unroll
            for (int q = 0; q < 2; q++) {
                const float4 m = *reinterpret_cast<const float4*>(&s_mu[16 * j + 8 * half + 4 * q]);
                const float mv[4] = {m.x, m.y, m.z, m.w};
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    const float v = raw[q][i] - mv[i];
                    n2 = __builtin_fmaf(v, v, n2);
                    const _Float16 vh = (_Float16)v;
                    xh[4 * q + i] = vh;
                    xl[4 * q + i] = (_Float16)__builtin_fmaf((float)vh, -2048.f, v * 2048.f);  // 2^11 (v - vh), exact
                }
            }
#pragma unroll
            for (int kt = 0; kt < NCT; kt++) {
                // (a truncated basis' zero rows are multiplied like any others: their coefficients come out zero)
                const halfx8 th = __builtin_bit_cast(halfx8, basis16[((kt * NJ + j) * 2) * 64 + lane]);
                const halfx8 tl = __builtin_bit_cast(halfx8, basis16[((kt * NJ + j) * 2 + 1) * 64 + lane]);
                am[kt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(th, xh, j ? am[kt] : zero, 0, 0, 0);
                ac[kt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(th, xl, j ? ac[kt] : zero, 0, 0, 0);
                ac[kt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(tl, xh, ac[kt], 0, 0, 0);
            }
            // (steps stay apart in the schedule: merged, their operands would not fit the registers of two wavefronts
            // per SIMD)
            __builtin_amdgcn_sched_barrier(0);
        };
        // Pair pr of this tile sits in buffer A or B as (pr odd) != SWAP says; a buffer is requested again as soon as
        // its steps are converted: for the pair two further on, which past this tile's end is pair 0 or 1 of the next
        // tile (whose SWAP is this one's for an even number of pairs and the opposite for an odd one, so that pair
        // finds its data where it looks for it).
#pragma unroll
        for (int pr = 0; pr < NP; pr++) {
            const bool in_b = ((pr & 1) != 0) != SWAP;
#pragma unroll
            for (int u = 0; u < 2; u++) {
                const int j = 2 * pr + u;
                if (j < NJ && j < NJA) {  // wavefront-uniform
                    if (in_b) step(j, bufB[u]); else step(j, bufA[u]);
                }
            }
            const int npr = pr + 2;
            if (npr < NP) {
                if (in_b) load_pair(tile, npr, bufB); else load_pair(tile, npr, bufA);
            } else if (next_tile < p.n_tiles && npr - NP < NP) {
                if (in_b) load_pair(next_tile, npr - NP, bufB); else load_pair(next_tile, npr - NP, bufA);
            }
        }
        n2 += __shfl_xor(n2, 32, 64);  // the other half of the pixel
        const bool force = !(n2 < 1.0e9f);  // too large for f16 (or not finite): every coefficient decided exactly
        const float tau = fminf(fmaxf(p.kappa * __builtin_sqrtf(n2), p.tau_min), 0.125f);
        const float near_limit = force ? -1.f : 0.5f - tau;

#pragma unroll
        for (int kt = 0; kt < NCT; kt++) {
            const bool k_ok = kt * 32 + 16 * half < C && px_ok;  // (C a multiple of 16: a lane's 16 coefficients all in or all out)
            uint32_t word[4], ub[16];
            float maxd = 0.f;
#pragma unroll
            for (int r = 0; r < 16; r++) {
                const float t = __builtin_fmaf(ac[kt][r], inv_delta_lo, am[kt][r] * inv_delta);
                const float u = t + magic;  // round half to even
                maxd = fmaxf(maxd, fabsf(t - (u - magic)));
                ub[r] = clamp_pattern(u, magic_lo, magic_hi);
                if (k_ok) hist_add(ub[r]);
            }
#pragma unroll
            for (int g = 0; g < 4; g++)
                word[g] = __builtin_amdgcn_perm(__builtin_amdgcn_perm(ub[4 * g + 3], ub[4 * g + 2], 0x0c0c0400u),
                                                __builtin_amdgcn_perm(ub[4 * g + 1], ub[4 * g], 0x0c0c0400u), 0x05040100u);
            if (k_ok)
                *reinterpret_cast<uint4*>(p.syms + px * C + kt * 32 + 16 * half) = make_uint4(word[0], word[1], word[2], word[3]);
            if (__builtin_expect(__any(!(maxd <= near_limit) && k_ok), 0)) {
                // the values too close to a rounding boundary go to the wavefront's list (resolved when it is full
                // and after the last tile)
                uint32_t near_mask = 0;
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    const float t = __builtin_fmaf(ac[kt][r], inv_delta_lo, am[kt][r] * inv_delta);
                    if (!(fabsf(t - __builtin_rintf(t)) <= near_limit) && k_ok) near_mask |= 1u << r;
                }
                const int k0 = kt * 32 + 16 * half;
                const uint32_t incoming = wave_sum((uint32_t)__popc(near_mask));
                if (*fix_count + incoming > (uint32_t)kFixList) resolve_list();
                if (incoming > (uint32_t)kFixList) {
#pragma unroll 1
                    for (int r = 0; r < 16; r++) {
                        if ((near_mask >> r) & 1u) {
                            const uint32_t slot = atomicAdd(fix_count, 1u);
                            fix_list[slot] = (uint32_t)(k0 + r) | ((uint32_t)l32 << 8) |
                                             (((word[r >> 2] >> (8 * (r & 3))) & 255u) << 13);
                            fix_tile[slot] = (uint32_t)tile;
                        }
                        wave_sync_lds();
                        resolve_list();
                    }
                } else {
                    while (near_mask) {
                        const int r = __ffs((int)near_mask) - 1;
                        near_mask &= near_mask - 1;
                        uint32_t sy = 0;
#pragma unroll
                        for (int g = 0; g < 4; g++)
                            if (g == (r >> 2)) sy = (word[g] >> (8 * (r & 3))) & 255u;
                        const uint32_t slot = atomicAdd(fix_count, 1u);
                        fix_list[slot] = (uint32_t)(k0 + r) | ((uint32_t)l32 << 8) | (sy << 13);
                        fix_tile[slot] = (uint32_t)tile;
                    }
                    wave_sync_lds();
                }
            }
        }
    };
    if constexpr ((NP & 1) != 0) {
        for (;;) {
            if (tile >= p.n_tiles) break;
            tile_body(std::false_type{}, tile);
            tile += stride;
            if (tile >= p.n_tiles) break;
            tile_body(std::true_type{}, tile);
            tile += stride;
        }
    } else {
        for (; tile < p.n_tiles; tile += stride) tile_body(std::false_type{}, tile);
    }
    if (*fix_count) resolve_list();
    __syncthreads();
    for (int row = tid; row < WAVES * K; row += THREADS) {
        const uint4* r4 = reinterpret_cast<const uint4*>(whist + (size_t)row * kHistLanes);
        uint32_t total = 0;
#pragma unroll
        for (int q = 0; q < kHistLanes / 4; q++) {
            const uint4 v = r4[q];
            total += (v.x + v.y) + (v.z + v.w);
        }
        s_red[row] = total;
    }
    __syncthreads();
    if (tid < K) {
        uint32_t total = 0;
#pragma unroll
        for (int q = 0; q < WAVES; q++) total += s_red[q * K + tid];
        p.hist_parts[(size_t)blockIdx.x * K + tid] = total;
    }
}

static hipError_t launch_rows(const BasisDevice& b, const float* d_x, int64_t P, int64_t HW, int layout, float delta,
                              int bits, uint8_t* d_syms, const CoderScratch& cs, int* n_parts, hipStream_t s) {
    RowParams p{};
    p.x = d_x;
    p.basis16 = b.fwd16;
    p.mu = b.mu;
    p.Trow = b.T;
    p.P = P;
    p.HW = HW;
    p.C = b.C;
    p.bits = bits;
    p.active_tiles = (b.active_rows + 31) / 32;
    p.inv_delta = (float)(1.0 / (double)delta);
    p.delta = delta;
    // The fast pass is off by at most about 2^-22 sum |T[k][c]| |x[c] - mu[c]| (three representation errors of
    // 2^-22 each and the fp32 accumulation) <= |T[k]|_2 |x - mu|_2 times that; values closer than 8 times this
    // (in steps) to a rounding boundary are decided in fp64 instead.  The floor covers the rounding of the
    // scaled value itself (magnitude up to 2^(b-1)).
    p.kappa = 1.9073486e-6f /* 2^-19 */ * b.row_norm * p.inv_delta;
    p.tau_min = 4.7683716e-7f /* 2^-21 */ * (float)(1 << (bits - 1));
    p.n_tiles = (P + 31) / 32;
    p.syms = d_syms;
    p.hist_parts = cs.hist_parts;
    p.ctrl = cs.ctrl;
    p.lookback = cs.lookback;
    p.n_groups = cs.n_groups;
    p.pk = PackParams{};
    if (!p.x || !p.basis16 || !p.mu || !p.Trow || !p.syms || !p.hist_parts || !p.ctrl || !p.lookback)
        return hipErrorInvalidValue;  // (a field left out would be a wild pointer on the device)
    const int nct = b.Cpad / 32;
    // eight wavefronts on one copy of the basis where two four-wavefront workgroups (each with its own copy) do not
    // fit a compute unit's LDS and there are tiles enough for them
    // (measured at 128 channels, 25.7 M values: 67 us against 62 us with four wavefronts, one per SIMD -- the second
    // wavefront's registers do not fit without spills -- so the eight-wavefront form stays off)
    const bool vec0 = (b.C % 4) == 0;
    // 128 channels: eight wavefronts on one copy of the basis, two per SIMD, each working tile by tile with one pair
    // of accumulators (two four-wavefront workgroups with a copy each would not fit a compute unit's LDS).  Measured
    // at 25.7 M values: 57 us against 63 us with four wavefronts, one per SIMD.  (The same form for 144 channels
    // spills registers: 119 us against 80 us.)
    // (planar tensors: the loads' addresses do not fit the registers either; 8 bits: eight wavefronts' histograms do
    // not fit LDS beside the basis)
    auto lds_for = [&](int wv) {
        return sizeof(float) * (size_t)b.Cpad * b.Cpad + sizeof(uint32_t) * wv * kHistLanes * ((size_t)1 << bits);
    };
    const bool eight = nct == 4 && layout == FMTC_NHWC && p.n_tiles > 1024 && lds_for(8) <= 144 * 1024;
    const int waves = eight ? 8 : 4;
    const size_t lds = lds_for(waves);
    // workgroups a compute unit holds at once: by registers (rows_waves_per_simd) and by LDS
    const size_t lds_static = (size_t)waves * (2 * kFixList + 1 + 256) * 4 + (size_t)nct * 128 + 512;
    int per_cu = eight ? 1 : rows_waves_per_simd(nct, false, 4);
    const int by_lds = (int)((160 * 1024) / (lds + lds_static));
    if (per_cu > by_lds) per_cu = by_lds < 1 ? 1 : by_lds;
    int64_t gx = (p.n_tiles + waves - 1) / waves;
    const int64_t cap = 256 * (int64_t)per_cu;
    if (gx > cap) gx = cap;
    *n_parts = (int)gx;
    const bool vec = vec0;
    hipError_t el = hipSuccess;
    // Four and five coefficient tiles, channels last, a multiple of 16 channels: the streaming form, four wavefronts.
    // (Measured: 144 channels, 28.9 M values, 79 -> 62 us; 128 channels, 3.2 M values, 15.9 -> 13.6 us.  With more
    // tiles than SIMDs at four coefficient tiles the eight-wavefront form of k_project_quantize_rows below stays: 50 us
    // at 25.7 M values against 53 us for this kernel with four wavefronts and 48 to 58 us with eight, whose registers
    // fit or spill with the compiler's schedule.)
    if ((nct == 5 || (nct == 4 && !eight)) && layout == FMTC_NHWC && (b.C % 16) == 0) {
        const int swaves = 4;
        const bool whole = b.C == nct * 32;  // else 16 channels less
        const size_t slds = lds_for(swaves);
        int64_t sgx = (p.n_tiles + swaves - 1) / swaves;
        if (sgx > 256) sgx = 256;  // one workgroup per compute unit (the basis takes 64 to 100 KB of its LDS)
        *n_parts = (int)sgx;
#define FMTC_STREAM_J(NCT, WV, NJA)                                                                              \
    do {                                                                                                         \
        hipError_t ea = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_project_quantize_stream<NCT, WV, NJA>), \
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)slds);             \
        if (ea != hipSuccess) return ea;                                                                         \
        el = launch(K_PROJECT, k_project_quantize_stream<NCT, WV, NJA>, dim3((unsigned)sgx), dim3(WV * 64), slds, s, p); \
    } while (0)
#define FMTC_STREAM(NCT, WV)                                                                                     \
    do {                                                                                                         \
        if (whole) FMTC_STREAM_J(NCT, WV, 2 * NCT); else FMTC_STREAM_J(NCT, WV, 2 * NCT - 1);                    \
    } while (0)
        if (nct == 5) FMTC_STREAM(5, 4);
        else FMTC_STREAM(4, 4);
#undef FMTC_STREAM_J
#undef FMTC_STREAM
        return el;
    }
#define FMTC_ROWS_W(NCT, LAY, VEC, WV)                                                                           \
    do {                                                                                                         \
        if (lds > 32 * 1024) {                                                                                   \
            hipError_t ea = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_project_quantize_rows<NCT, LAY, VEC, false, WV>), \
                                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);          \
            if (ea != hipSuccess) return ea;                                                                     \
        }                                                                                                        \
        el = launch(K_PROJECT, k_project_quantize_rows<NCT, LAY, VEC, false, WV>, dim3((unsigned)gx), dim3(WV * 64), lds, s, p); \
    } while (0)
#define FMTC_ROWS(NCT, LAY, VEC) FMTC_ROWS_W(NCT, LAY, VEC, 4)
#define FMTC_ROWS_N(LAY, VEC)                                                                                    \
    do {                                                                                                         \
        if (nct == 1) FMTC_ROWS(1, LAY, VEC);                                                                    \
        else if (nct == 2) FMTC_ROWS(2, LAY, VEC);                                                               \
        else if (nct == 3) FMTC_ROWS(3, LAY, VEC);                                                               \
        else FMTC_ROWS(4, LAY, VEC);                                                                             \
    } while (0)
    if (eight) {
        if (vec) FMTC_ROWS_W(4, FMTC_NHWC, true, 8); else FMTC_ROWS_W(4, FMTC_NHWC, false, 8);
    } else if (nct == 5) {  // channels-last only (see launch_project_quantize)
        if (vec) FMTC_ROWS(5, FMTC_NHWC, true); else FMTC_ROWS(5, FMTC_NHWC, false);
    } else if (layout == FMTC_NHWC) { if (vec) FMTC_ROWS_N(FMTC_NHWC, true); else FMTC_ROWS_N(FMTC_NHWC, false); }
    else                            { if (vec) FMTC_ROWS_N(FMTC_NCHW, true); else FMTC_ROWS_N(FMTC_NCHW, false); }
#undef FMTC_ROWS_N
#undef FMTC_ROWS
#undef FMTC_ROWS_W
    return el;
}

// The fused kernel for a channel count and layout, its LDS size, and how many of its workgroups the device
// holds at once (0: shape not supported or the query failed).
static int fused_kernel_for(int C, int layout, const void** fn_out, size_t* lds_out) {
    if (!(C == 32 || C == 64 || C == 128)) return 0;
    const int nct = C / 32;
    const size_t lds = sizeof(float) * (size_t)C * C + 4 * 4096 + sizeof(PackShared);
    const void* fn = nullptr;
#define FMTC_FUSED(NCT, LAY) fn = reinterpret_cast<const void*>(&k_project_quantize_rows<NCT, LAY, true, true>)
    if (layout == FMTC_NHWC) {
        if (nct == 1) FMTC_FUSED(1, FMTC_NHWC); else if (nct == 2) FMTC_FUSED(2, FMTC_NHWC); else FMTC_FUSED(4, FMTC_NHWC);
    } else {
        if (nct == 1) FMTC_FUSED(1, FMTC_NCHW); else if (nct == 2) FMTC_FUSED(2, FMTC_NCHW); else FMTC_FUSED(4, FMTC_NCHW);
    }
#undef FMTC_FUSED
    *fn_out = fn;
    *lds_out = lds;
    static std::atomic<int> resident[2][3];  // (zero-initialised; every thread computes the same values)
    std::atomic<int>& slot = resident[layout == FMTC_NHWC][nct == 4 ? 2 : nct - 1];
    int cap = slot.load(std::memory_order_relaxed);
    if (!cap) {
        int dev = 0, cus = 0, per_cu = 0;
        if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess ||
            hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, 256, lds) != hipSuccess || cus < 1 || per_cu < 1)
            return 0;
        cap = cus;  // one workgroup per compute unit, whatever more would fit
        slot.store(cap, std::memory_order_relaxed);
    }
    return cap;
}

// The one-kernel encoder is used where every chunk group gets a workgroup of its own: its workgroups work through
// their groups in lock step (project, pack, wait for the position, store), which is the shortest path for a
// tensor the device holds at once and loses to two specialised kernels beyond that (measured: 25 us against
// 17 + 10 us at 196 groups, 135 us against 60 + 40 us at 1568).
bool encode_static_fused_applies(int C, int layout, uint32_t chunk_syms, uint32_t n_groups) {
    const void* fn;
    size_t lds;
    if (chunk_syms != 4096u) return false;
    const int cap = fused_kernel_for(C, layout, &fn, &lds);
    return cap > 0 && n_groups <= (uint32_t)cap;
}

// Projection, quantizer and packing with a table fixed beforehand as one kernel.  Returns hipErrorNotSupported
// where encode_static_fused_applies() says no.
hipError_t launch_encode_static_fused(const BasisDevice& b, const float* d_x, int64_t N, int64_t HW, int layout,
                                      float delta, int bits, const CoderScratch& cs, const PackParams& pk,
                                      hipStream_t s) {
    const int64_t P = N * HW;
    const void* fn = nullptr;
    size_t lds = 0;
    const int cap = fused_kernel_for(b.C, layout, &fn, &lds);
    if (cap <= 0 || pk.chunk_syms != 4096u || pk.n_groups > (uint32_t)cap) return hipErrorNotSupported;
    RowParams p{};
    p.x = d_x;
    p.basis16 = b.fwd16;
    p.mu = b.mu;
    p.Trow = b.T;
    p.P = P;
    p.HW = HW;
    p.C = b.C;
    p.bits = bits;
    p.active_tiles = (b.active_rows + 31) / 32;
    p.inv_delta = (float)(1.0 / (double)delta);
    p.delta = delta;
    p.kappa = 1.9073486e-6f /* 2^-19 */ * b.row_norm * p.inv_delta;  // see launch_rows
    p.tau_min = 4.7683716e-7f /* 2^-21 */ * (float)(1 << (bits - 1));
    p.n_tiles = (P + 31) / 32;
    p.syms = nullptr;
    p.hist_parts = nullptr;
    p.ctrl = cs.ctrl;
    p.lookback = cs.lookback;
    p.n_groups = cs.n_groups;
    p.pk = pk;
    if (!p.x || !p.basis16 || !p.mu || !p.Trow || !p.ctrl || !p.lookback || !pk.enc_table || !pk.stream || !pk.lookback ||
        !pk.ctrl)
        return hipErrorInvalidValue;  // (a field left out would be a wild pointer on the device)
    const uint32_t grid = pk.n_groups < (uint32_t)cap ? pk.n_groups : (uint32_t)cap;
    void* args[] = {(void*)&p};
    hipEvent_t ev_a = nullptr, ev_b = nullptr;
    if (prof_next(K_PROJECT, &ev_a, &ev_b))
        return hipExtLaunchKernel(fn, dim3(grid), dim3(256), args, lds, s, ev_a, ev_b, 0);
    return hipLaunchKernel(fn, dim3(grid), dim3(256), args, lds, s);
}

// ---------------------------------------------------------------------------
// Wide tensors whose channel count is a multiple of 16: the projection as a tiled matrix product.
// A pixel's channels fit neither a wavefront's registers nor (for more than a few pixels) LDS, so
// the contraction index is cut instead.  A workgroup owns a tile of 128 coefficients x 128 pixels
// (each of its 4 wavefronts 64 x 64: 2 x 2 matrix tiles with two accumulators each) and walks the
// channels 16 at a time.  What a step needs goes from L2 / HBM straight into a ring of three LDS
// slots, two steps ahead of its use and with no registers in between:
//   basis   8 KB in operand order (wavefront w: both f16 parts of coefficient tile w);
//   pixels  8 KB of fp32 as they lie in the tensor: thread (pixel, h) of wavefront w its channels
//           [16 s + 8 h, + 8) of pixel 32 w + pixel -- exactly the operand entry of its lane.
// One step ahead of the matrix instructions every thread reads its own eight values back,
// removes the mean, cuts them in their two f16 parts and writes them as pixel operands into one
// of two LDS buffers; one barrier per step hands a slot and a buffer over.
// Every operand byte read from LDS feeds two matrix tiles, every basis byte from L2 four pixel
// tiles -- what the kernel that holds whole pixels in LDS lacks.  The waits count loads in flight
// (they complete in order), so every wavefront issues the same loads in the same order whatever
// part of its tile lies outside the tensor: addresses are clamped, values zeroed.  Quantizer,
// histogram, stores and exact decisions as in the narrow-tensor kernel: a lane ends up with 16
// consecutive coefficients of its pixel.
// ---------------------------------------------------------------------------
struct GemmParams {
    const float* x;
    const uint4* basis16;  // fwd16 packing: [ncs][NJ][2][64]
    const float* mu;       // [Cpad]
    const float* Trow;
    int64_t P, HW;
    int C, ncs, NJ, bits;
    int64_t n_pt, n_ptg;   // 32-pixel tiles, groups of four of them
    float inv_delta, delta, kappa, tau_min;
    int hist_shift;
    uint8_t* syms;
    uint32_t* hist_parts;
    CoderCtrl* ctrl;
    unsigned long long* lookback;
    uint32_t n_groups;
};

constexpr int kGemmFix = 64;  // values per wavefront waiting for their exact decision

template <int LAYOUT>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_project_quantize_gemm4(GemmParams p) {
    __shared__ __align__(16) uint4 stageA[3][8][64];     // per 16-channel step: (coefficient tile, part), operand order
    __shared__ __align__(16) uint4 stageX[3][4][2][64];  // per step: fp32 pixels as loaded, [wavefront][instruction][lane]
    __shared__ __align__(16) uint4 stageB[2][4][2][64];  // per step: (pixel tile, part), operand order
    __shared__ float s_n2[4][32];
    __shared__ uint32_t s_fix_a[4][kGemmFix], s_fix_px[4][kGemmFix], s_fix_count[4];
    extern __shared__ __align__(16) uint8_t dyn_lds[];    // mean [Cpad], then histogram copies [4][K << HS]
    constexpr int XL = LAYOUT == FMTC_NHWC ? 2 : 8;       // transfers of one step's pixels per wavefront
    constexpr int LD = 2 + XL;                            // ... of one step in all (basis: 2)

    zero_coder_scratch(p.ctrl, p.lookback, p.n_groups);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, l32 = lane & 31;
    const int C = p.C, NJ = p.NJ, K = 1 << p.bits, HS = p.hist_shift, HC = 1 << HS;
    const int ktp = wave & 1, ptp = wave >> 1;  // this wavefront's pair of coefficient tiles / pixel tiles
    const int kt0 = blockIdx.y * 4;
    float* s_mu = reinterpret_cast<float*>(dyn_lds);
    uint32_t* whist = reinterpret_cast<uint32_t*>(dyn_lds) + 16 * NJ;
    for (int i = tid; i < 4 * K * HC; i += 256) whist[i] = 0u;
    for (int i = tid; i < 16 * NJ; i += 256) s_mu[i] = p.mu[i];
    uint32_t* wh0 = whist + wave * K * HC;
    uint32_t* wh = wh0 + (lane & (HC - 1));
    uint32_t* fix_a = s_fix_a[wave];
    uint32_t* fix_px = s_fix_px[wave];
    uint32_t* fix_count = &s_fix_count[wave];
    if (lane == 0) *fix_count = 0u;
    __syncthreads();

    const int zero_sym = 1 << (p.bits - 1);
    const float lo = (float)(-zero_sym), hi = (float)(zero_sym - 1), zero_f = (float)zero_sym;
    const float inv_delta = p.inv_delta, inv_delta_lo = p.inv_delta * (1.f / 2048.f);

    // exact fp64 decision of the listed values, four per round (one per 16-lane group)
    auto resolve_list = [&]() {
        __builtin_amdgcn_s_waitcnt(0x0F70);  // the symbols that get patched have been stored
        const uint32_t n = (uint32_t)__builtin_amdgcn_readfirstlane((int)*fix_count);
        for (uint32_t base = 0; base < n; base += 4) {
            const uint32_t idx = base + (uint32_t)(lane >> 4);
            const bool active = idx < n;
            const uint32_t e = active ? fix_a[idx] : 0u;
            const int k = (int)(e & 0xffffu);
            const uint32_t old = e >> 16;
            const int64_t qpx = active ? (int64_t)fix_px[idx] : 0;
            int64_t xbase, xstride;
            if constexpr (LAYOUT == FMTC_NHWC) {
                xbase = qpx * C;
                xstride = 1;
            } else {
                const int64_t n_img = qpx / p.HW;
                xbase = n_img * (int64_t)C * p.HW + (qpx - n_img * p.HW);
                xstride = p.HW;
            }
            double part = 0.0;
            if (active)
#pragma unroll 8  // independent loads of eight terms in flight together: the loop is all latency
                for (int c = lane & 15; c < C; c += 16)
                    part += (double)p.Trow[(size_t)k * C + c] * ((double)p.x[xbase + c * xstride] - (double)p.mu[c]);
#pragma unroll
            for (int o = 8; o > 0; o >>= 1) part += __shfl_xor(part, o, 64);  // stays inside the 16-lane group
            double qd = rint(part / (double)p.delta);
            qd = fmin(fmax(qd, (double)lo), (double)hi);
            const uint32_t sfix = (uint32_t)((int)qd + zero_sym);
            if (active && (lane & 15) == 0 && sfix != old) {
                atomicSub(&wh0[old << HS], 1u);
                atomicAdd(&wh0[sfix << HS], 1u);
                p.syms[qpx * C + k] = (uint8_t)sfix;
            }
        }
        wave_sync_lds();
        if (lane == 0) *fix_count = 0u;
        wave_sync_lds();
    };

    for (int64_t ptg = blockIdx.x; ptg < p.n_ptg; ptg += gridDim.x) {
        const int64_t pt0 = ptg * 4;
        floatx16 am[2][2], ac[2][2];
#pragma unroll
        for (int a = 0; a < 2; a++)
#pragma unroll
            for (int b = 0; b < 2; b++)
#pragma unroll
                for (int r = 0; r < 16; r++) { am[a][b][r] = 0.f; ac[a][b][r] = 0.f; }

        // this thread's pixel (of pixel tile pt0 + wave); past the end of the tensor the last pixel is loaded
        // in its place and zeroed on conversion
        const int64_t px_raw = (pt0 + wave) * 32 + l32;
        const bool px_ok = px_raw < p.P;
        const int64_t px_ld = px_ok ? px_raw : p.P - 1;
        int64_t xbase, xstride;
        if constexpr (LAYOUT == FMTC_NHWC) {
            xbase = px_ld * C;
            xstride = 1;
        } else {
            const int64_t n_img = px_ld / p.HW;
            xbase = n_img * (int64_t)C * p.HW + (px_ld - n_img * p.HW);
            xstride = p.HW;
        }
        int kt_ld = kt0 + wave;
        kt_ld = kt_ld < p.ncs ? kt_ld : p.ncs - 1;  // a tile past the end repeats the last one; its results are dropped
        const uint4* a_src = p.basis16 + (size_t)kt_ld * NJ * 128 + lane;
        // Everything step s needs, on its way into ring slot s % 3: both parts of basis tile kt0 + wave, and
        // channels [16 s + 8 h, + 8) of this thread's pixel -- the operand entry of lane (pixel, h).  Steps past the
        // end repeat the last one, so that every wavefront always has the same number of loads in flight.
        auto issue = [&](int s) {
            const int slot = s % 3;
            s = s < NJ ? s : NJ - 1;
            load_to_lds<16>(a_src + (size_t)s * 128, &stageA[slot][2 * wave][0]);
            load_to_lds<16>(a_src + (size_t)s * 128 + 64, &stageA[slot][2 * wave + 1][0]);
            int c0 = 16 * s + 8 * half;
            c0 = c0 < C ? c0 : 0;  // C is a multiple of 16: all eight channels or none (then zeroed on conversion)
            if constexpr (LAYOUT == FMTC_NHWC) {
                const float* src = p.x + xbase + c0;
                load_to_lds<16>(src, &stageX[slot][wave][0][0]);
                load_to_lds<16>(src + 4, &stageX[slot][wave][1][0]);
            } else {
#pragma unroll
                for (int e = 0; e < 8; e++)
                    load_to_lds<4>(p.x + xbase + (int64_t)(c0 + e) * xstride,
                                   reinterpret_cast<uint32_t*>(&stageX[slot][wave][0][0]) + 64 * e);
            }
        };
        float n2 = 0.f;
        // this thread's eight channels of step s: mean removed, cut in two f16 parts, written as pixel operands
        auto convert = [&](int s) {
            const int c0 = 16 * s + 8 * half;
            const bool ok = px_ok && c0 < C;
            float v[8];
            if constexpr (LAYOUT == FMTC_NHWC) {
                const float4 a = *reinterpret_cast<const float4*>(&stageX[s % 3][wave][0][lane]);
                const float4 b = *reinterpret_cast<const float4*>(&stageX[s % 3][wave][1][lane]);
                v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
            } else {
                const float* raw = reinterpret_cast<const float*>(&stageX[s % 3][wave][0][0]) + lane;
#pragma unroll
                for (int e = 0; e < 8; e++) v[e] = raw[64 * e];
            }
            const float4 m0 = *reinterpret_cast<const float4*>(&s_mu[c0]);
            const float4 m1 = *reinterpret_cast<const float4*>(&s_mu[c0 + 4]);
            const float m[8] = {m0.x, m0.y, m0.z, m0.w, m1.x, m1.y, m1.z, m1.w};
            halfx8 vh, vl;
#pragma unroll
            for (int e = 0; e < 8; e++) {
                float d = ok ? v[e] - m[e] : 0.f;
                n2 = __builtin_fmaf(d, d, n2);
                // (no clamp of values beyond f16: what their infinities make of the products stays in the pixel's own
                // column of outputs, and such a pixel is decided exactly in all coefficients, see n2)
                const _Float16 h = (_Float16)d;
                vh[e] = h;
                vl[e] = (_Float16)__builtin_fmaf((float)h, -2048.f, d * 2048.f);  // 2^11 (d - h), exact, one mixed multiply-add
            }
            stageB[s & 1][wave][0][lane] = __builtin_bit_cast(uint4, vh);
            stageB[s & 1][wave][1][lane] = __builtin_bit_cast(uint4, vl);
        };

        issue(0);
        issue(1);
        wait_loads<LD>();  // step 0 has landed (this wavefront's part)
        convert(0);
        for (int s = 0; s < NJ; s++) {
            // in flight: step s (unless s = 0) and step s + 1
            wait_loads<LD>();  // step s has landed
            __syncthreads();  // everybody's part of it, and everybody's pixel operands of step s; slot of step s - 1 is free
            issue(s + 2);
            const uint4(*sa)[64] = stageA[s % 3];
            halfx8 th[2], tl[2], xh[2], xl[2];
#pragma unroll
            for (int a = 0; a < 2; a++) {
                th[a] = __builtin_bit_cast(halfx8, sa[(2 * ktp + a) * 2][lane]);
                tl[a] = __builtin_bit_cast(halfx8, sa[(2 * ktp + a) * 2 + 1][lane]);
                xh[a] = __builtin_bit_cast(halfx8, stageB[s & 1][2 * ptp + a][0][lane]);
                xl[a] = __builtin_bit_cast(halfx8, stageB[s & 1][2 * ptp + a][1][lane]);
            }
#pragma unroll
            for (int a = 0; a < 2; a++)
#pragma unroll
                for (int b = 0; b < 2; b++) {
                    am[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(th[a], xh[b], am[a][b], 0, 0, 0);
                    ac[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(th[a], xl[b], ac[a][b], 0, 0, 0);
                }
#pragma unroll
            for (int a = 0; a < 2; a++)
#pragma unroll
                for (int b = 0; b < 2; b++)
                    ac[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(tl[a], xh[b], ac[a][b], 0, 0, 0);
            wait_loads<LD>();  // step s + 1 has landed
            if (s + 1 < NJ) convert(s + 1);  // into the operand buffer step s - 1 read, free since the barrier above
        }
        wait_loads<0>();  // the repeated loads of the last steps too
        n2 += __shfl_xor(n2, 32, 64);
        if (half == 0) s_n2[wave][l32] = n2;
        __syncthreads();  // all wavefronts are done with the stages: the next group's first loads may overwrite them

        // ---- quantizer, histogram, stores: accumulator r of lane (pixel, h) is coefficient kt*32 + 16h + r ----
#pragma unroll
        for (int b = 0; b < 2; b++) {
            const int64_t pt = pt0 + 2 * ptp + b;
            if (pt >= p.n_pt) continue;  // wavefront-uniform
            const int64_t px = pt * 32 + l32;
            const bool out_ok = px < p.P;
            const float pn2 = s_n2[2 * ptp + b][l32];
            const bool force = !(pn2 < 1.0e9f);  // too large for f16, or not finite: every coefficient decided exactly
            const float tau = fminf(fmaxf(p.kappa * __builtin_sqrtf(pn2), p.tau_min), 0.125f);
            const float near_limit = force ? -1.f : 0.5f - tau;
#pragma unroll
            for (int a = 0; a < 2; a++) {
                const int kt = kt0 + 2 * ktp + a;
                if (kt >= p.ncs) continue;  // wavefront-uniform
                const int k0 = kt * 32 + 16 * half;
                const bool ok = out_ok && k0 < C;  // C is a multiple of 16: all sixteen coefficients or none
                uint32_t word[4] = {0u, 0u, 0u, 0u};
                uint32_t near_mask = 0;
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    const float t = __builtin_fmaf(ac[a][b][r], inv_delta_lo, am[a][b][r] * inv_delta);
                    const float q = __builtin_rintf(t);  // round half to even
                    if (!(fabsf(t - q) <= near_limit)) near_mask |= 1u << r;
                    const float qc = __builtin_amdgcn_fmed3f(q, lo, hi) + zero_f;  // clamped level, as a symbol
                    word[r >> 2] = __builtin_amdgcn_cvt_pk_u8_f32(qc, r & 3, word[r >> 2]);
                    if (ok) atomicAdd(&wh[((uint32_t)qc < (uint32_t)K ? (uint32_t)qc : (uint32_t)(K - 1)) << HS], 1u);  // (in range whatever qc is)
                }
                if (ok)
                    *reinterpret_cast<uint4*>(p.syms + px * C + k0) = make_uint4(word[0], word[1], word[2], word[3]);
                if (!ok) near_mask = 0;
                if (__builtin_expect(__any(near_mask != 0), 0)) {
                    // note the flagged values; the list is resolved when it could overflow and at the end
#pragma unroll 1
                    for (int r = 0; r < 16; r++) {
                        const bool f = (near_mask >> r) & 1u;
                        const uint32_t incoming = (uint32_t)__popcll(__ballot(f));
                        if (incoming == 0) continue;
                        if (*fix_count + incoming > (uint32_t)kGemmFix) resolve_list();
                        if (f) {
                            const uint32_t slot = atomicAdd(fix_count, 1u);
                            fix_a[slot] = (uint32_t)(k0 + r) | (((word[r >> 2] >> (8 * (r & 3))) & 255u) << 16);
                            fix_px[slot] = (uint32_t)px;
                        }
                        wave_sync_lds();
                    }
                }
            }
        }
        if (*fix_count) resolve_list();  // before the next group's loads: the waits there count loads in flight
    }
    __syncthreads();
    // one row of partial counts per workgroup (see the narrow-tensor kernel); the operand buffers are free now
    uint32_t* s_red = reinterpret_cast<uint32_t*>(&stageA[0][0][0]);
    for (int row = tid; row < 4 * K; row += 256) {
        uint32_t total = 0;
        for (int q = 0; q < HC; q++) total += whist[((size_t)row << HS) + q];
        s_red[row] = total;
    }
    __syncthreads();
    if (tid < K)
        p.hist_parts[(size_t)(blockIdx.y * gridDim.x + blockIdx.x) * K + tid] =
            (s_red[tid] + s_red[K + tid]) + (s_red[2 * K + tid] + s_red[3 * K + tid]);
}

// The same product with 8 wavefronts per 128 x 128 tile, two per SIMD, each 2 coefficient tiles x 1 pixel tile and a
// quarter of the conversion work: while one wavefront of a SIMD converts, the other's matrix instructions run.  More
// LDS operand reads per matrix instruction and one workgroup per compute unit: the faster form for tensors whose
// tiles all fit the device at once (measured C = 960: 57 -> 47 us, C = 512 at N = 64: 33 -> 26 us), the slower one
// beyond (N = 256, C = 256: 49 -> 61 us).
template <int LAYOUT>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_project_quantize_gemm8(GemmParams p) {
    __shared__ __align__(16) uint4 stageA[3][8][64];     // per 16-channel step: (coefficient tile, part), operand order
    __shared__ __align__(16) uint4 stageX[3][8][64];     // per step: fp32 pixels as loaded, [wavefront][lane] (16 bytes each)
    __shared__ __align__(16) uint4 stageB[2][4][2][64];  // per step: (pixel tile, part), operand order
    __shared__ float s_n2[4][32];
    __shared__ uint32_t s_fix_a[8][kGemmFix], s_fix_px[8][kGemmFix], s_fix_count[8];
    extern __shared__ __align__(16) uint8_t dyn_lds[];    // mean [Cpad], then histogram copies [8][K << HS]
    constexpr int XL = LAYOUT == FMTC_NHWC ? 1 : 4;       // transfers of one step's pixels per wavefront
    constexpr int LD = 1 + XL;                            // ... of one step in all (basis: 1)

    zero_coder_scratch(p.ctrl, p.lookback, p.n_groups);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, l32 = lane & 31;
    const int C = p.C, NJ = p.NJ, K = 1 << p.bits, HS = p.hist_shift, HC = 1 << HS;
    // 8 wavefronts, two per SIMD (one converts while the other's matrix instructions run): wavefront w owns the
    // pair ktp of coefficient tiles and pixel tile xpt, and brings quarter xq of the 16 channels of xpt's pixels
    const int ktp = wave & 1, xpt = wave >> 1, xq = 2 * (wave & 1) + half;
    const int kt0 = blockIdx.y * 4;
    float* s_mu = reinterpret_cast<float*>(dyn_lds);
    uint32_t* whist = reinterpret_cast<uint32_t*>(dyn_lds) + 16 * NJ;
    for (int i = tid; i < 8 * K * HC; i += 512) whist[i] = 0u;
    for (int i = tid; i < 16 * NJ; i += 512) s_mu[i] = p.mu[i];
    uint32_t* wh0 = whist + wave * K * HC;
    uint32_t* wh = wh0 + (lane & (HC - 1));
    uint32_t* fix_a = s_fix_a[wave];
    uint32_t* fix_px = s_fix_px[wave];
    uint32_t* fix_count = &s_fix_count[wave];
    if (lane == 0) *fix_count = 0u;
    __syncthreads();

    const int zero_sym = 1 << (p.bits - 1);
    const float lo = (float)(-zero_sym), hi = (float)(zero_sym - 1), zero_f = (float)zero_sym;
    const float inv_delta = p.inv_delta, inv_delta_lo = p.inv_delta * (1.f / 2048.f);

    // exact fp64 decision of the listed values, four per round (one per 16-lane group)
    auto resolve_list = [&]() {
        __builtin_amdgcn_s_waitcnt(0x0F70);  // the symbols that get patched have been stored
        const uint32_t n = (uint32_t)__builtin_amdgcn_readfirstlane((int)*fix_count);
        for (uint32_t base = 0; base < n; base += 4) {
            const uint32_t idx = base + (uint32_t)(lane >> 4);
            const bool active = idx < n;
            const uint32_t e = active ? fix_a[idx] : 0u;
            const int k = (int)(e & 0xffffu);
            const uint32_t old = e >> 16;
            const int64_t qpx = active ? (int64_t)fix_px[idx] : 0;
            int64_t xbase, xstride;
            if constexpr (LAYOUT == FMTC_NHWC) {
                xbase = qpx * C;
                xstride = 1;
            } else {
                const int64_t n_img = qpx / p.HW;
                xbase = n_img * (int64_t)C * p.HW + (qpx - n_img * p.HW);
                xstride = p.HW;
            }
            double part = 0.0;
            if (active)
#pragma unroll 8  // independent loads of eight terms in flight together: the loop is all latency
                for (int c = lane & 15; c < C; c += 16)
                    part += (double)p.Trow[(size_t)k * C + c] * ((double)p.x[xbase + c * xstride] - (double)p.mu[c]);
#pragma unroll
            for (int o = 8; o > 0; o >>= 1) part += __shfl_xor(part, o, 64);  // stays inside the 16-lane group
            double qd = rint(part / (double)p.delta);
            qd = fmin(fmax(qd, (double)lo), (double)hi);
            const uint32_t sfix = (uint32_t)((int)qd + zero_sym);
            if (active && (lane & 15) == 0 && sfix != old) {
                atomicSub(&wh0[old << HS], 1u);
                atomicAdd(&wh0[sfix << HS], 1u);
                p.syms[qpx * C + k] = (uint8_t)sfix;
            }
        }
        wave_sync_lds();
        if (lane == 0) *fix_count = 0u;
        wave_sync_lds();
    };

    for (int64_t ptg = blockIdx.x; ptg < p.n_ptg; ptg += gridDim.x) {
        const int64_t pt0 = ptg * 4;
        floatx16 am[2], ac[2];
#pragma unroll
        for (int a = 0; a < 2; a++)
#pragma unroll
            for (int r = 0; r < 16; r++) { am[a][r] = 0.f; ac[a][r] = 0.f; }

        // this thread's pixel (of pixel tile pt0 + xpt); past the end of the tensor the last pixel is loaded
        // in its place and zeroed on conversion
        const int64_t px_raw = (pt0 + xpt) * 32 + l32;
        const bool px_ok = px_raw < p.P;
        const int64_t px_ld = px_ok ? px_raw : p.P - 1;
        int64_t xbase, xstride;
        if constexpr (LAYOUT == FMTC_NHWC) {
            xbase = px_ld * C;
            xstride = 1;
        } else {
            const int64_t n_img = px_ld / p.HW;
            xbase = n_img * (int64_t)C * p.HW + (px_ld - n_img * p.HW);
            xstride = p.HW;
        }
        int kt_ld = kt0 + (wave >> 1);
        kt_ld = kt_ld < p.ncs ? kt_ld : p.ncs - 1;  // a tile past the end repeats the last one; its results are dropped
        const uint4* a_src = p.basis16 + ((size_t)kt_ld * NJ * 2 + (wave & 1)) * 64 + lane;
        // Everything step s needs, on its way into ring slot s % 3: part wave % 2 of basis tile kt0 + wave / 2, and
        // channels [16 s + 4 xq, + 4) of this thread's pixel -- half of an operand entry.  Steps past the end
        // repeat the last one, so that every wavefront always has the same number of loads in flight.
        auto issue = [&](int s) {
            const int slot = s % 3;
            s = s < NJ ? s : NJ - 1;
            load_to_lds<16>(a_src + (size_t)s * 128, &stageA[slot][wave][0]);
            int c0 = 16 * s + 4 * xq;
            c0 = c0 < C ? c0 : 0;  // C is a multiple of 16: all four channels or none (then zeroed on conversion)
            if constexpr (LAYOUT == FMTC_NHWC) {
                load_to_lds<16>(p.x + xbase + c0, &stageX[slot][wave][0]);
            } else {
#pragma unroll
                for (int e = 0; e < 4; e++)
                    load_to_lds<4>(p.x + xbase + (int64_t)(c0 + e) * xstride,
                                   reinterpret_cast<uint32_t*>(&stageX[slot][wave][0]) + 64 * e);
            }
        };
        float n2 = 0.f;
        // this thread's four channels of step s: mean removed, cut in two f16 parts, written into the pixel
        // operands (entry of lane (pixel, xq / 2), elements 4 (xq % 2) .. + 3)
        typedef _Float16 halfx4 __attribute__((ext_vector_type(4)));
        auto convert = [&](int s) {
            const int c0 = 16 * s + 4 * xq;
            const bool ok = px_ok && c0 < C;
            float v[4];
            if constexpr (LAYOUT == FMTC_NHWC) {
                const float4 a = *reinterpret_cast<const float4*>(&stageX[s % 3][wave][lane]);
                v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
            } else {
                const float* raw = reinterpret_cast<const float*>(&stageX[s % 3][wave][0]) + lane;
#pragma unroll
                for (int e = 0; e < 4; e++) v[e] = raw[64 * e];
            }
            const float4 m0 = *reinterpret_cast<const float4*>(&s_mu[c0]);
            const float m[4] = {m0.x, m0.y, m0.z, m0.w};
            halfx4 vh, vl;
#pragma unroll
            for (int e = 0; e < 4; e++) {
                float d = ok ? v[e] - m[e] : 0.f;
                n2 = __builtin_fmaf(d, d, n2);
                // (no clamp of values beyond f16: what their infinities make of the products stays in the pixel's own
                // column of outputs, and such a pixel is decided exactly in all coefficients, see n2)
                const _Float16 h = (_Float16)d;
                vh[e] = h;
                vl[e] = (_Float16)__builtin_fmaf((float)h, -2048.f, d * 2048.f);  // 2^11 (d - h), exact, one mixed multiply-add
            }
            uint2* dst = reinterpret_cast<uint2*>(&stageB[s & 1][xpt][0][l32 + 32 * (xq >> 1)]) + (xq & 1);
            dst[0] = __builtin_bit_cast(uint2, vh);
            dst[128] = __builtin_bit_cast(uint2, vl);  // part 1: 64 entries of 16 bytes further on
        };

        issue(0);
        issue(1);
        wait_loads<LD>();  // step 0 has landed (this wavefront's part)
        convert(0);
        for (int s = 0; s < NJ; s++) {
            // in flight: step s (unless s = 0) and step s + 1
            wait_loads<LD>();  // step s has landed
            __syncthreads();  // everybody's part of it, and everybody's pixel operands of step s; slot of step s - 1 is free
            if (s == 0 && tid < 128) s_n2[tid >> 5][tid & 31] = 0.f;  // everybody has left the previous group's epilogue
            issue(s + 2);
            const uint4(*sa)[64] = stageA[s % 3];
            halfx8 th[2], tl[2];
#pragma unroll
            for (int a = 0; a < 2; a++) {
                th[a] = __builtin_bit_cast(halfx8, sa[(2 * ktp + a) * 2][lane]);
                tl[a] = __builtin_bit_cast(halfx8, sa[(2 * ktp + a) * 2 + 1][lane]);
            }
            const halfx8 xh = __builtin_bit_cast(halfx8, stageB[s & 1][xpt][0][lane]);
            const halfx8 xl = __builtin_bit_cast(halfx8, stageB[s & 1][xpt][1][lane]);
#pragma unroll
            for (int a = 0; a < 2; a++) {
                am[a] = __builtin_amdgcn_mfma_f32_32x32x16_f16(th[a], xh, am[a], 0, 0, 0);
                ac[a] = __builtin_amdgcn_mfma_f32_32x32x16_f16(th[a], xl, ac[a], 0, 0, 0);
            }
#pragma unroll
            for (int a = 0; a < 2; a++) ac[a] = __builtin_amdgcn_mfma_f32_32x32x16_f16(tl[a], xh, ac[a], 0, 0, 0);
            wait_loads<LD>();  // step s + 1 has landed
            if (s + 1 < NJ) convert(s + 1);  // into the operand buffer step s - 1 read, free since the barrier above
        }
        wait_loads<0>();  // the repeated loads of the last steps too
        // a pixel's sum of squares: its four quarters sit in two lanes of each of two wavefronts
        n2 += __shfl_xor(n2, 32, 64);
        if (half == 0) atomicAdd(&s_n2[xpt][l32], n2);
        __syncthreads();  // all wavefronts are done with the stages: the next group's first loads may overwrite them

        // ---- quantizer, histogram, stores: accumulator r of lane (pixel, h) is coefficient kt*32 + 16h + r ----
        {
            const int64_t pt = pt0 + xpt;
            if (pt < p.n_pt) {  // wavefront-uniform
            const int64_t px = pt * 32 + l32;
            const bool out_ok = px < p.P;
            const float pn2 = s_n2[xpt][l32];
            const bool force = !(pn2 < 1.0e9f);  // too large for f16, or not finite: every coefficient decided exactly
            const float tau = fminf(fmaxf(p.kappa * __builtin_sqrtf(pn2), p.tau_min), 0.125f);
            const float near_limit = force ? -1.f : 0.5f - tau;
#pragma unroll
            for (int a = 0; a < 2; a++) {
                const int kt = kt0 + 2 * ktp + a;
                if (kt >= p.ncs) continue;  // wavefront-uniform
                const int k0 = kt * 32 + 16 * half;
                const bool ok = out_ok && k0 < C;  // C is a multiple of 16: all sixteen coefficients or none
                uint32_t word[4] = {0u, 0u, 0u, 0u};
                uint32_t near_mask = 0;
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    const float t = __builtin_fmaf(ac[a][r], inv_delta_lo, am[a][r] * inv_delta);
                    const float q = __builtin_rintf(t);  // round half to even
                    if (!(fabsf(t - q) <= near_limit)) near_mask |= 1u << r;
                    const float qc = __builtin_amdgcn_fmed3f(q, lo, hi) + zero_f;  // clamped level, as a symbol
                    word[r >> 2] = __builtin_amdgcn_cvt_pk_u8_f32(qc, r & 3, word[r >> 2]);
                    if (ok) atomicAdd(&wh[((uint32_t)qc < (uint32_t)K ? (uint32_t)qc : (uint32_t)(K - 1)) << HS], 1u);  // (in range whatever qc is)
                }
                if (ok)
                    *reinterpret_cast<uint4*>(p.syms + px * C + k0) = make_uint4(word[0], word[1], word[2], word[3]);
                if (!ok) near_mask = 0;
                if (__builtin_expect(__any(near_mask != 0), 0)) {
                    // note the flagged values; the list is resolved when it could overflow and at the end
#pragma unroll 1
                    for (int r = 0; r < 16; r++) {
                        const bool f = (near_mask >> r) & 1u;
                        const uint32_t incoming = (uint32_t)__popcll(__ballot(f));
                        if (incoming == 0) continue;
                        if (*fix_count + incoming > (uint32_t)kGemmFix) resolve_list();
                        if (f) {
                            const uint32_t slot = atomicAdd(fix_count, 1u);
                            fix_a[slot] = (uint32_t)(k0 + r) | (((word[r >> 2] >> (8 * (r & 3))) & 255u) << 16);
                            fix_px[slot] = (uint32_t)px;
                        }
                        wave_sync_lds();
                    }
                }
            }
        }
        }
        if (*fix_count) resolve_list();  // before the next group's loads: the waits there count loads in flight
    }
    __syncthreads();
    // one row of partial counts per workgroup (see the narrow-tensor kernel); the operand buffers are free now
    uint32_t* s_red = reinterpret_cast<uint32_t*>(&stageA[0][0][0]);
    for (int row = tid; row < 8 * K; row += 512) {
        uint32_t total = 0;
        for (int q = 0; q < HC; q++) total += whist[((size_t)row << HS) + q];
        s_red[row] = total;
    }
    __syncthreads();
    if (tid < K)
        p.hist_parts[(size_t)(blockIdx.y * gridDim.x + blockIdx.x) * K + tid] =
            ((s_red[tid] + s_red[K + tid]) + (s_red[2 * K + tid] + s_red[3 * K + tid])) +
            ((s_red[4 * K + tid] + s_red[5 * K + tid]) + (s_red[6 * K + tid] + s_red[7 * K + tid]));
}

// Columns [c0, C) of the symbols [P][C] set to one value (c0 and C multiples of 16), and one row of partial
// counts that says so: what the tiled projection leaves out when the basis' last rows are all zero (a truncated
// basis: those coefficients are 0, their symbol the zero level).
__global__ __launch_bounds__(256) void k_fill_symbol_columns(uint8_t* __restrict__ syms, int64_t P, int C, int c0,
                                                             uint32_t value, int bits, uint32_t* __restrict__ hist_row) {
    const uint32_t v4 = value * 0x01010101u;
    const int64_t per_px = (C - c0) / 16;
    const int64_t n = P * per_px;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
        const int64_t px = i / per_px, j = i - px * per_px;
        *reinterpret_cast<uint4*>(syms + (size_t)px * (size_t)C + (size_t)c0 + 16 * (size_t)j) = make_uint4(v4, v4, v4, v4);
    }
    if (blockIdx.x == 0 && (int)threadIdx.x < (1 << bits))
        hist_row[threadIdx.x] = threadIdx.x == value ? (uint32_t)(P * (int64_t)(C - c0)) : 0u;
}

static hipError_t launch_gemm(const BasisDevice& b, const float* d_x, int64_t P, int64_t HW, int layout, float delta,
                              int bits, uint8_t* d_syms, const CoderScratch& cs, int* n_parts, hipStream_t s) {
    const int ncs = b.Cpad / 32, NJ = b.Cpad / 16;
    const int64_t n_pt = (P + 31) / 32;
    GemmParams p{};
    p.x = d_x;
    p.basis16 = reinterpret_cast<const uint4*>(b.fwd16);
    p.mu = b.mu;
    p.Trow = b.T;
    p.P = P;
    p.HW = HW;
    p.C = b.C;
    p.ncs = ncs;
    p.NJ = NJ;
    p.bits = bits;
    p.n_pt = n_pt;
    p.n_ptg = (n_pt + 3) / 4;
    p.inv_delta = (float)(1.0 / (double)delta);
    p.delta = delta;
    p.kappa = 1.9073486e-6f /* 2^-19 */ * b.row_norm * p.inv_delta;  // see launch_rows
    p.tau_min = 4.7683716e-7f /* 2^-21 */ * (float)(1 << (bits - 1));
    p.syms = d_syms;
    p.hist_parts = cs.hist_parts;
    p.ctrl = cs.ctrl;
    p.lookback = cs.lookback;
    p.n_groups = cs.n_groups;
    // every pointer the kernel follows is set (a field left out here would be a wild pointer on the device)
    if (!p.x || !p.basis16 || !p.mu || !p.Trow || !p.syms || !p.hist_parts || !p.ctrl || !p.lookback)
        return hipErrorInvalidValue;
    // groups of four coefficient tiles; those whose rows of the basis are all zero (truncation) are not computed:
    // k_fill_symbol_columns writes their symbols and counts
    const int gy_all = (ncs + 3) / 4;
    int gy = ((b.active_rows + 31) / 32 + 3) / 4;
    gy = gy < 1 ? 1 : (gy > gy_all ? gy_all : gy);
    int64_t gx = p.n_ptg;
    if (gx * gy_all > kMaxHistParts) gx = kMaxHistParts / gy_all;
    *n_parts = (int)(gx * gy) + (gy < gy_all ? 1 : 0);
    if (gy < gy_all) {
        const int c0 = gy * 128;  // < C, and C - c0 is a multiple of 16 like C
        const int64_t pieces = P * ((b.C - c0) / 16);
        int64_t blocks = (pieces + 255) / 256;
        blocks = blocks > 2048 ? 2048 : blocks;
        hipLaunchKernelGGL(k_fill_symbol_columns, dim3((unsigned)blocks), dim3(256), 0, s, d_syms, P, b.C, c0,
                           (uint32_t)(1 << (bits - 1)), bits, cs.hist_parts + (size_t)(gx * gy) * ((size_t)1 << bits));
        hipError_t ef = hipGetLastError();
        if (ef != hipSuccess) return ef;
    }
    // 8 wavefronts per tile while every tile has a compute unit of its own, 4 (two workgroups per compute unit) beyond
    const bool eight = p.n_ptg * gy <= 256;
    const int waves = eight ? 8 : 4;
    // histogram copies per wavefront: as many as 2 KB of LDS hold, 16 at most, 2 at least
    int copies = 512 >> bits;
    copies = copies >= 16 ? 16 : (copies >= 8 ? 8 : (copies >= 4 ? 4 : 2));
    p.hist_shift = copies == 16 ? 4 : (copies == 8 ? 3 : (copies == 4 ? 2 : 1));
    const size_t lds = sizeof(float) * b.Cpad + sizeof(uint32_t) * waves * copies * ((size_t)1 << bits);
    dim3 grid((unsigned)gx, (unsigned)gy);
    if (eight)
        return layout == FMTC_NHWC
                   ? launch(K_PROJECT, k_project_quantize_gemm8<FMTC_NHWC>, grid, dim3(512), lds, s, p)
                   : launch(K_PROJECT, k_project_quantize_gemm8<FMTC_NCHW>, grid, dim3(512), lds, s, p);
    return layout == FMTC_NHWC
               ? launch(K_PROJECT, k_project_quantize_gemm4<FMTC_NHWC>, grid, dim3(256), lds, s, p)
               : launch(K_PROJECT, k_project_quantize_gemm4<FMTC_NCHW>, grid, dim3(256), lds, s, p);
}

hipError_t launch_project_quantize(const BasisDevice& b, const float* d_x, int64_t N, int64_t HW, int layout,
                                   float delta, int bits, uint8_t* d_syms, const CoderScratch& cs, int* n_parts,
                                   hipStream_t s) {
    const int64_t P = N * HW;
    // 160 padded channels still fit the one-wavefront-per-32-pixels kernel for channels-last tensors (planar
    // loads take more registers than it has left)
    if (b.Cpad <= 128 || (b.Cpad == 160 && layout == FMTC_NHWC))
        return launch_rows(b, d_x, P, HW, layout, delta, bits, d_syms, cs, n_parts, s);
    // wide: the tiled matrix product needs whole groups of 16 channels; other channel counts keep the pixel-tile kernel
    if (b.C % 16 == 0) return launch_gemm(b, d_x, P, HW, layout, delta, bits, d_syms, cs, n_parts, s);
    return launch_wide(b, d_x, P, HW, layout, delta, bits, d_syms, cs, n_parts, s);
}

// Histogram of given symbols (staged coder entry point): one row of partial counts per workgroup.
// Values outside the alphabet are not counted.
__global__ __launch_bounds__(256) void k_histogram(const uint8_t* __restrict__ syms, uint64_t V, int bits,
                                                   uint32_t* __restrict__ hist_parts, CoderCtrl* ctrl,
                                                   unsigned long long* lookback, uint32_t n_groups) {
    __shared__ uint32_t lhist[256];
    zero_coder_scratch(ctrl, lookback, n_groups);
    lhist[threadIdx.x] = 0u;
    __syncthreads();
    const unsigned K = 1u << bits;
    for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < V; i += (uint64_t)gridDim.x * 256) {
        unsigned sy = syms[i];
        if (sy < K) atomicAdd(&lhist[sy], 1u);
    }
    __syncthreads();
    if (threadIdx.x < K) hist_parts[(size_t)blockIdx.x * K + threadIdx.x] = lhist[threadIdx.x];
}

hipError_t launch_histogram(const uint8_t* d_syms, uint64_t V, int bits, const CoderScratch& cs, int* n_parts,
                            hipStream_t s) {
    uint64_t want = (V + 256 * 16 - 1) / (256 * 16);
    unsigned blocks = (unsigned)(want < 1 ? 1 : (want > (uint64_t)kMaxHistParts ? (uint64_t)kMaxHistParts : want));
    *n_parts = (int)blocks;
    return launch(K_HISTOGRAM, k_histogram, dim3(blocks), dim3(256), 0, s, d_syms, V, bits, cs.hist_parts, cs.ctrl,
                  cs.lookback, cs.n_groups);
}

}  // namespace fmtc
