// 8-bit basis and 8-bit activations (paper section 3.1 "Linear transform": the PCA matrix is stored at 8 bits;
// section 5: the hardware moves 8-bit activations).  Both contractions run on the integer matrix cores
// (v_mfma_i32_32x32x16_i8) and are exact; every rounding decision is one fp64 operation on exact operands, so the
// results are defined bit for bit:
//   forward  n = 256 sum_c Tq[k][c] xq[c] - sum_c Tq[k][c] mf[c],  level = rne(n * g),  g = s_T s_x / (256 Delta)
//   inverse  m = sum_k Tq[k][c] (s[k] - 2^(b-1)),  v = fma(m, h, mf[c]),  xq^ = clamp(rne(v / 256), 0, 255),
//            h = 256 s_T Delta / s_x   (computed as rne(fma(m, h / 256, mf[c] / 256)): scaling by 2^-8 is exact)
// The matrix instruction multiplies signed bytes; unsigned activations and symbols enter as (value - 128) (one XOR)
// and the difference is folded into per-row integer offsets prepared with the basis.
//
// One wavefront owns 32 pixels.  Operand order (both operands): lane l holds row/pixel l % 32 and the 8 bytes
// 16 s + 8 (l / 32) .. + 7 of contraction step s.  The rows of a 32-row tile of the basis are stored permuted so
// that a lane's 16 results are 16 consecutive coefficients (channels): one 16-byte store.
#include "fmtc_internal.h"

namespace fmtc {

typedef int v16i __attribute__((ext_vector_type(16)));

// 8 consecutive bytes row[c0 .. c0 + 7] of a row-major byte matrix with rows of n_cols bytes; zeros outside.
// wide: n_cols is a multiple of 8 and base is 8-byte aligned, so the group is either whole or absent.
__device__ __forceinline__ unsigned long long load8_row(const uint8_t* __restrict__ base, int64_t row, int64_t n_rows,
                                                        int c0, int n_cols, bool wide) {
    if (row >= n_rows || c0 >= n_cols) return 0ull;
    const uint8_t* q = base + (size_t)row * (size_t)n_cols + (size_t)c0;
    if (wide) return *reinterpret_cast<const unsigned long long*>(q);
    unsigned long long v = 0ull;
#pragma unroll
    for (int e = 0; e < 8; e++)
        if (c0 + e < n_cols) v |= (unsigned long long)q[e] << (8 * e);
    return v;
}

// the same bytes of pixel p from a planar (n, c, hw) tensor
__device__ __forceinline__ unsigned long long load8_planar(const uint8_t* __restrict__ base, int64_t p, int64_t P,
                                                           int c0, int C, int64_t HW) {
    if (p >= P || c0 >= C) return 0ull;
    const int64_t n = p / HW, hw = p - n * HW;
    const uint8_t* q = base + ((size_t)n * (size_t)C + (size_t)c0) * (size_t)HW + (size_t)hw;
    unsigned long long v = 0ull;
#pragma unroll
    for (int e = 0; e < 8; e++)
        if (c0 + e < C) v |= (unsigned long long)q[(size_t)e * (size_t)HW] << (8 * e);
    return v;
}

struct Int8Params {
    const uint8_t* in;              // forward: activations in `layout`; inverse: symbols [P][C]
    uint8_t* out;                   // forward: symbols [P][C]; inverse: activations in `layout`
    const unsigned long long* op8;  // [nct][NS][64] basis (forward) or its transpose (inverse), operand order
    const double* row_off;          // forward [nct * 32]: sum_c Tq[k][c] (mf[c] - 256 * 128), an integer below 2^53
    const int* col_sum;             // inverse [nct * 32]: sum_k Tq[k][c]
    const double* mean_d;           // inverse [nct * 32]: the mean in activation units (mean_fix / 256, exact)
    int64_t P, HW, n_tiles;
    int C, NS, nct, bits;
    double factor;                  // g (forward) or h / 256 (inverse)
    // forward, whole encoder only (else null): one partial histogram per workgroup [gridDim.x][2^bits], and the
    // coder's scratch that the first kernel of a call clears
    uint32_t* hist_parts;
    CoderCtrl* ctrl;
    unsigned long long* lookback;
    uint32_t n_groups;
};

constexpr int kCopies = 16;  // histogram copies per wavefront
constexpr unsigned long long kFlip = 0x8080808080808080ull;  // unsigned byte -> (value - 128) as a signed byte

// NSR > 0: the pixel tile's operand (NS <= NSR steps) stays in registers over the coefficient tiles;
// NSR == 0: it is loaded again for every coefficient tile (wide tensors).
template <int LAYOUT, int NSR, bool INVERSE>
__global__ __launch_bounds__(256) void k_int8_tiles(Int8Params p) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int C = p.C, NS = p.NS;
    const int hk = 1 << (p.bits - 1);
    const bool wide = (C % 8) == 0;
    // Histogram (forward, whole encoder), in dynamic LDS: kCopies interleaved copies per wavefront (bin s of copy q
    // at word s * kCopies + q, lane l counts in copy l % kCopies), because most symbols of a tile are the same few
    // values and one copy would serialise the lanes on a few words.
    // The basis operand of narrow tensors (NSR > 0: at most 8 steps, 16 KB) is copied into LDS first; wide ones read
    // it from global memory through the cache.
    extern __shared__ __align__(16) uint32_t s_dyn[];  // basis operand [nct][NS][64] x 8 bytes if NSR > 0, then
                                                       // the histogram [4][K * kCopies] if hist
    const int basis_words = NSR > 0 ? p.nct * NS * 128 : 0;
    uint32_t* s_hist = s_dyn + basis_words;
    const bool hist = !INVERSE && p.hist_parts != nullptr;
    const int K = 1 << p.bits;
    uint32_t* wh = s_hist + (size_t)wave * K * kCopies + (lane & (kCopies - 1));
    if (NSR > 0) {
        const uint4* src = reinterpret_cast<const uint4*>(p.op8);
        uint4* dst = reinterpret_cast<uint4*>(s_dyn);
        for (int i = threadIdx.x; i < basis_words / 4; i += 256) dst[i] = src[i];
    }
    if (hist) {
        zero_coder_scratch(p.ctrl, p.lookback, p.n_groups);
        for (int i = threadIdx.x; i < 4 * K * kCopies; i += 256) s_hist[i] = 0u;
    }
    if (NSR > 0 || hist) __syncthreads();
    const unsigned long long* op8 = NSR > 0 ? reinterpret_cast<const unsigned long long*>(s_dyn) : p.op8;
    for (int64_t tile = (int64_t)blockIdx.x * 4 + wave; tile < p.n_tiles; tile += (int64_t)gridDim.x * 4) {
        const int64_t px = tile * 32 + l32;
        auto operand = [&](int s) -> long {
            const int c0 = 16 * s + 8 * half;
            unsigned long long v;
            if (INVERSE || LAYOUT == FMTC_NHWC) v = load8_row(p.in, px, p.P, c0, C, wide);
            else v = load8_planar(p.in, px, p.P, c0, C, p.HW);
            return (long)(v ^ kFlip);
        };
        long b[NSR > 0 ? NSR : 1];
        if (NSR > 0) {
#pragma unroll
            for (int s = 0; s < NSR; s++) b[s] = s < NS ? operand(s) : 0l;
        }
        for (int kt = 0; kt < p.nct; kt++) {
            v16i acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
            const unsigned long long* a8 = op8 + ((size_t)kt * NS) * 64 + lane;
            if (NSR > 0) {
#pragma unroll
                for (int s = 0; s < NSR; s++)
                    if (s < NS) acc = __builtin_amdgcn_mfma_i32_32x32x16_i8((long)a8[(size_t)s * 64], b[s], acc, 0, 0, 0);
            } else {
                for (int s = 0; s < NS; s++)
                    acc = __builtin_amdgcn_mfma_i32_32x32x16_i8((long)a8[(size_t)s * 64], operand(s), acc, 0, 0, 0);
            }
            // this lane: pixel px, results r0 .. r0 + 15 (coefficients, or channels for the inverse)
            const int r0 = kt * 32 + 16 * half;
            // (all integers below 2^53, so the fp64 operations before the one rounding product are exact)
            uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int v = 0; v < 16; v++) {
                const int r = r0 + v;  // < nct * 32: the per-row arrays are padded to that
                double t;
                if (!INVERSE) {
                    const double n = fma((double)acc[v], 256.0, -p.row_off[r]);
                    t = fmin(fmax(rint(n * p.factor), (double)-hk), (double)(hk - 1)) + (double)hk;
                } else {
                    const int m = acc[v] + (128 - hk) * p.col_sum[r];
                    t = fmin(fmax(rint(fma((double)m, p.factor, p.mean_d[r])), 0.0), 255.0);
                }
                w[v >> 2] |= (uint32_t)(int)t << (8 * (v & 3));
            }
            if (hist && px < p.P) {
                if (r0 + 16 <= C) {
#pragma unroll
                    for (int v = 0; v < 16; v++) atomicAdd(&wh[((w[v >> 2] >> (8 * (v & 3))) & 0xffu) * kCopies], 1u);
                } else {
#pragma unroll
                    for (int v = 0; v < 16; v++)
                        if (r0 + v < C) atomicAdd(&wh[((w[v >> 2] >> (8 * (v & 3))) & 0xffu) * kCopies], 1u);
                }
            }
            if (px < p.P && r0 < C) {
                if (INVERSE && LAYOUT == FMTC_NCHW) {
                    const int64_t n = px / p.HW, hw = px - n * p.HW;
#pragma unroll
                    for (int v = 0; v < 16; v++)
                        if (r0 + v < C)
                            p.out[((size_t)n * (size_t)C + (size_t)(r0 + v)) * (size_t)p.HW + (size_t)hw] =
                                (uint8_t)(w[v >> 2] >> (8 * (v & 3)));
                } else {
                    uint8_t* q = p.out + (size_t)px * (size_t)C + (size_t)r0;
                    if ((C % 16) == 0) {
                        *reinterpret_cast<uint4*>(q) = make_uint4(w[0], w[1], w[2], w[3]);
                    } else {
#pragma unroll
                        for (int v = 0; v < 16; v++)
                            if (r0 + v < C) q[v] = (uint8_t)(w[v >> 2] >> (8 * (v & 3)));
                    }
                }
            }
        }
    }
    if (hist) {
        __syncthreads();
        if ((int)threadIdx.x < K) {
            uint32_t sum = 0;
            for (int q = 0; q < 4; q++)
                for (int c = 0; c < kCopies; c++) sum += s_hist[((size_t)q * K + threadIdx.x) * kCopies + c];
            p.hist_parts[(size_t)blockIdx.x * K + threadIdx.x] = sum;
        }
    }
}

template <bool INVERSE>
static hipError_t launch_int8(int kernel_id, const Int8Params& p, int layout, int* n_parts, hipStream_t s) {
    if (!p.in || !p.out || !p.op8 || (!INVERSE && !p.row_off) || (INVERSE && (!p.col_sum || !p.mean_d)))
        return hipErrorInvalidValue;
    if (p.P < 1 || p.C < 1 || p.C > 1024 || p.NS != (p.C + 15) / 16 || p.nct != (p.C + 31) / 32 || p.HW < 1 ||
        p.n_tiles != (p.P + 31) / 32 || p.bits < 2 || p.bits > 8)
        return hipErrorInvalidValue;
    if (p.hist_parts && (INVERSE || !p.ctrl || !p.lookback)) return hipErrorInvalidValue;
    int64_t gx = (p.n_tiles + 3) / 4;
    const int64_t cap = p.hist_parts ? kMaxHistParts : 2048;  // one histogram row per workgroup
    if (gx > cap) gx = cap;
    if (n_parts) *n_parts = (int)gx;
    const dim3 grid((unsigned)gx), block(256);
    const size_t lds = (p.NS <= 8 ? (size_t)p.nct * p.NS * 512 : 0) +  // the basis operand of the NSR = 8 kernels
                       (p.hist_parts ? sizeof(uint32_t) * 4 * kCopies * ((size_t)1 << p.bits) : 0);
    const bool planar = layout == FMTC_NCHW;  // of the activations: read by the forward kernel, written by the inverse
#define FMTC_INT8(LAY, NSR)                                                                                     \
    do {                                                                                                        \
        if (lds > 32 * 1024) {                                                                                  \
            hipError_t ea = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_int8_tiles<LAY, NSR, INVERSE>), \
                                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);          \
            if (ea != hipSuccess) return ea;                                                                    \
        }                                                                                                       \
        return launch(kernel_id, k_int8_tiles<LAY, NSR, INVERSE>, grid, block, lds, s, p);                      \
    } while (0)
    if (p.NS <= 8) {
        if (planar) FMTC_INT8(FMTC_NCHW, 8);
        FMTC_INT8(FMTC_NHWC, 8);
    }
    if (planar) FMTC_INT8(FMTC_NCHW, 0);
    FMTC_INT8(FMTC_NHWC, 0);
#undef FMTC_INT8
}

hipError_t launch_quantize_u8(const Basis8Device& b, const uint8_t* d_xq, int64_t P, int64_t HW, int layout,
                              int bits, double g, uint8_t* d_syms, const CoderScratch* cs, int* n_parts,
                              hipStream_t s) {
    Int8Params p{};
    p.in = d_xq;
    p.out = d_syms;
    p.op8 = b.fwd8;
    p.row_off = b.row_off;
    p.col_sum = nullptr;
    p.mean_d = nullptr;
    p.P = P;
    p.HW = HW;
    p.n_tiles = (P + 31) / 32;
    p.C = b.C;
    p.NS = (b.C + 15) / 16;
    p.nct = (b.C + 31) / 32;
    p.bits = bits;
    p.factor = g;
    if (cs) {
        p.hist_parts = cs->hist_parts;
        p.ctrl = cs->ctrl;
        p.lookback = cs->lookback;
        p.n_groups = cs->n_groups;
        if (!p.hist_parts || !n_parts) return hipErrorInvalidValue;
    }
    return launch_int8<false>(K_QUANTIZE_U8, p, layout, n_parts, s);
}

hipError_t launch_reconstruct_u8(const Basis8Device& b, const uint8_t* d_syms, int64_t P, int64_t HW, int layout,
                                 int bits, double h, uint8_t* d_xq_hat, hipStream_t s) {
    Int8Params p{};
    p.in = d_syms;
    p.out = d_xq_hat;
    p.op8 = b.inv8;
    p.row_off = nullptr;
    p.col_sum = b.col_sum;
    p.mean_d = b.mean_d;
    p.P = P;
    p.HW = HW;
    p.n_tiles = (P + 31) / 32;
    p.C = b.C;
    p.NS = (b.C + 15) / 16;
    p.nct = (b.C + 31) / 32;
    p.bits = bits;
    p.factor = h;
    return launch_int8<true>(K_RECONSTRUCT_U8, p, layout, nullptr, s);
}

}  // namespace fmtc
