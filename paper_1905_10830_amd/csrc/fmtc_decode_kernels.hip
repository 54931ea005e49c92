// Decoder (paper section 3: variable length decoder, inverse quantizer, inverse
// transform; section 3.1 "Implementation": levels scaled back to the transform
// domain, then the inverse PCA).  One fused kernel:
//   1. every workgroup validates the header and the code length table and builds
//      the canonical decode tables and a 2^10-entry lookup table in LDS;
//   2. per tile of G chunks: one wavefront per chunk, one lane per run of 64
//      symbols (bit offset = prefix sum of the stored run sizes) decodes into an
//      LDS symbol tile;
//   3. x_hat = T^T (Delta q) + mu on the fp32 matrix cores
//      (v_mfma_f32_32x32x2_f32): symbols are converted on the fly from LDS, the
//      basis comes pre-packed in operand order from global memory (L2 resident).
// Nothing outside [stream, stream + bytes) is read whatever the stream holds.
#include "fmtc_internal.h"

namespace fmtc {

typedef float floatx16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ uint32_t dec_wave_exclusive_scan(uint32_t v, int lane) {
    uint32_t incl = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        uint32_t t = __shfl_up(incl, o, 64);
        if (lane >= o) incl += t;
    }
    return incl - v;
}

// byte address of symbol n of the tile: every run of 64 symbols is followed by 4
// pad bytes so that the 64 lanes of a decoding wavefront hit different banks
__device__ __forceinline__ uint32_t sym_addr(uint32_t n) { return n + 4u * (n >> 6); }


// Decodes the `cnt` symbols of one run (one lane) starting at bit `start` of a chunk.
// STAGED: the chunk's words are in LDS (`pw`, two zero words behind them); otherwise they are read from
// global memory (`gw`), zero past the chunk's end.  Returns false if bits matched no code word.
template <bool STAGED, bool ALIGNED4>
__device__ __forceinline__ bool decode_run(const uint32_t* pw, const uint32_t* __restrict__ gw, uint32_t nwords,
                                           uint32_t start, uint32_t cnt, uint32_t nbase, const uint16_t* lut,
                                           const uint32_t* cnt_len, const uint32_t* first_rank,
                                           const uint64_t* first_code, const uint16_t* sorted_sym,
                                           uint8_t* symtile) {
    auto fetch = [&](uint32_t rel) -> uint64_t {
        if constexpr (STAGED) return (uint64_t)pw[rel < nwords + 1 ? rel : nwords + 1];
        else return (rel < nwords) ? (uint64_t)gw[rel] : 0ull;
    };
    // word index can not wrap: start <= 64 runs * 65535 bits
    uint32_t widx = start >> 5;
    uint64_t window = fetch(widx) | (fetch(widx + 1) << 32);
    widx += 2;
    window >>= (start & 31);
    uint32_t avail = 64 - (start & 31);
    uint64_t nxt = fetch(widx);
    bool ok = true;
    uint32_t word = 0;
    for (uint32_t i = 0; i < cnt; i++) {
        // refill without a branch: more than 32 valid bits before every lookup
        const bool need = avail <= 32;
        window |= need ? (nxt << (avail & 63)) : 0ull;
        avail += need ? 32u : 0u;
        widx += need ? 1u : 0u;
        nxt = fetch(widx);
        uint32_t e = lut[window & ((1u << kLutBits) - 1)];
        uint32_t len = e >> 8, sym = e & 255;
        if (len) {
            window >>= len;
            avail -= len;
        } else {
            // code longer than the table: canonical decoding bit by bit
            uint64_t code = 0;
            bool found = false;
            for (int l = 1; l <= kMaxLen; l++) {
                if (avail <= 32) {
                    window |= fetch(widx++) << avail;
                    avail += 32;
                }
                code = (code << 1) | (window & 1);
                window >>= 1;
                avail--;
                uint64_t f = first_code[l];
                uint32_t c = cnt_len[l];
                if (c && code >= f && code - f < c) {
                    sym = sorted_sym[first_rank[l] + (uint32_t)(code - f)];
                    found = true;
                    break;
                }
            }
            if (!found) { ok = false; sym = 0; }
            nxt = fetch(widx);
        }
        if constexpr (ALIGNED4) {
            word |= sym << (8 * (i & 3));
            if ((i & 3) == 3) {
                *reinterpret_cast<uint32_t*>(symtile + sym_addr(nbase + i - 3)) = word;
                word = 0;
            }
        } else {
            symtile[sym_addr(nbase + i)] = (uint8_t)sym;
        }
    }
    return ok;
}

struct DecodeParams {
    const uint8_t* stream;
    size_t bytes;
    int64_t P;
    int64_t HW;
    int C;
    int bits;
    int G;             // chunks per tile
    int ct_per_group;  // 32-channel output tiles per workgroup row (blockIdx.y)
    int ncs;           // Cpad / 32
    const float* Bpk;  // inverse operand, packed
    const float* mu;   // [Cpad]
    float* xhat;       // NULL in symbols-only mode
    uint8_t* syms_out; // non-NULL in symbols-only mode
    uint32_t* err;
};

constexpr int kPayWords = 1022;  // LDS copy of a chunk's payload: up to ~8 bits/symbol; larger chunks read global memory

template <int MT, int LAYOUT, bool ALIGNED4>
__global__ __launch_bounds__(256) void k_decode(DecodeParams p) {
    __shared__ uint16_t lut[1 << kLutBits];
    __shared__ uint8_t len_s[256];
    __shared__ uint16_t sorted_sym[256];
    __shared__ uint32_t cnt_len[kMaxLen + 2];
    __shared__ uint32_t first_rank[kMaxLen + 2];
    __shared__ uint64_t first_code[kMaxLen + 2];
    __shared__ unsigned long long kraft;
    __shared__ uint32_t n_used, bad_len;
    __shared__ uint32_t pay[4][kPayWords + 2];  // per wavefront: the chunk's payload words
    extern __shared__ __align__(16) uint8_t symtile[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wavefront-uniform by construction
    const int half = lane >> 5, l32 = lane & 31;
    const int C = p.C;
    const int K = 1 << p.bits;

    // ---- header ----
    if (p.bytes < (size_t)(kHeaderBytes + kLenTableBytes)) {
        if (tid == 0 && blockIdx.x == 0 && blockIdx.y == 0) atomicOr(p.err, FMTC_ERR_HEADER);
        return;
    }
    const Header hd = *reinterpret_cast<const Header*>(p.stream);
    const uint64_t ppc = hd.px_per_chunk;
    const uint64_t chunk_syms64 = ppc * (uint64_t)C;
    bool ok = hd.magic == kMagic && hd.version == 1 && hd.bits == p.bits && hd.C == (uint32_t)C &&
              hd.P == (uint64_t)p.P && hd.sub_syms == (uint32_t)kSubSyms && ppc >= 1 &&
              (chunk_syms64 <= 4096 || ppc == 1) && hd.delta > 0.f;
    uint32_t n_chunks = 0, spc = 0;
    size_t off_sub = 0, off_pay = 0;
    if (ok) {
        uint64_t nch = ((uint64_t)p.P + ppc - 1) / ppc;
        spc = (uint32_t)((chunk_syms64 + kSubSyms - 1) / kSubSyms);
        ok = nch == hd.n_chunks && spc == hd.subs_per_chunk;
        n_chunks = (uint32_t)nch;
        size_t off_co = kHeaderBytes + kLenTableBytes;
        off_sub = (off_co + 4 * ((size_t)nch + 1) + 15) & ~(size_t)15;
        off_pay = (off_sub + 2 * (size_t)nch * spc + 15) & ~(size_t)15;
        ok = ok && p.bytes >= off_pay && (p.bytes - off_pay) / 4 >= hd.payload_words && hd.payload_words <= 0xffffffffull;
    }
    if (!ok) {
        if (tid == 0 && blockIdx.x == 0 && blockIdx.y == 0) atomicOr(p.err, FMTC_ERR_HEADER);
        return;
    }
    const uint32_t chunk_syms = (uint32_t)chunk_syms64;
    const uint32_t payload_words = (uint32_t)hd.payload_words;
    const uint32_t* chunk_off = reinterpret_cast<const uint32_t*>(p.stream + kHeaderBytes + kLenTableBytes);
    const uint16_t* sub_bits = reinterpret_cast<const uint16_t*>(p.stream + off_sub);
    const uint32_t* payload = reinterpret_cast<const uint32_t*>(p.stream + off_pay);
    const uint64_t V = (uint64_t)p.P * (uint64_t)C;

    // ---- code tables ----
    if (tid <= kMaxLen + 1) cnt_len[tid] = 0;
    if (tid == 0) { kraft = 0ull; n_used = 0; bad_len = 0; }
    __syncthreads();
    const int my_len = p.stream[kHeaderBytes + tid];
    len_s[tid] = (uint8_t)my_len;
    if (my_len > kMaxLen || (tid >= K && my_len != 0)) atomicAdd(&bad_len, 1u);
    else if (my_len) {
        atomicAdd(&cnt_len[my_len], 1u);
        atomicAdd(&kraft, 1ull << (kMaxLen - my_len));
        atomicAdd(&n_used, 1u);
    }
    __syncthreads();
    {
        bool table_ok = bad_len == 0 && n_used >= 1 &&
                        (n_used == 1 ? cnt_len[1] == 1 : kraft == (1ull << kMaxLen));
        if (!table_ok) {
            if (tid == 0 && blockIdx.x == 0 && blockIdx.y == 0) atomicOr(p.err, FMTC_ERR_TABLE);
            return;
        }
    }
    if (tid >= 1 && tid <= kMaxLen) {
        // first code and first rank of every length: code(l) = sum_{j<l} count(j) << (l-j)
        uint64_t code = 0;
        uint32_t rank = 0;
        for (int j = 1; j < tid; j++) {
            uint32_t c = cnt_len[j];
            code += (uint64_t)c << (tid - j);
            rank += c;
        }
        first_code[tid] = code;
        first_rank[tid] = rank;
    }
    __syncthreads();
    if (my_len) {
        int before = 0;
        for (int t = 0; t < tid; t++) before += (len_s[t] == my_len) ? 1 : 0;
        sorted_sym[first_rank[my_len] + before] = (uint16_t)tid;
    }
    __syncthreads();
    {
        uint32_t fc[kLutBits + 1], cn[kLutBits + 1], fr[kLutBits + 1];
#pragma unroll
        for (int l = 1; l <= kLutBits; l++) {
            fc[l] = (uint32_t)first_code[l];
            cn[l] = cnt_len[l];
            fr[l] = first_rank[l];
        }
        for (int idx = tid; idx < (1 << kLutBits); idx += 256) {
            uint32_t code = 0, hit_len = 0, hit_rank = 0;
#pragma unroll
            for (int l = 1; l <= kLutBits; l++) {
                code = (code << 1) | ((idx >> (l - 1)) & 1);
                bool hit = hit_len == 0 && code >= fc[l] && code - fc[l] < cn[l];
                hit_rank = hit ? fr[l] + code - fc[l] : hit_rank;
                hit_len = hit ? (uint32_t)l : hit_len;
            }
            lut[idx] = hit_len ? (uint16_t)(sorted_sym[hit_rank] | (hit_len << 8)) : (uint16_t)0;
        }
    }
    __syncthreads();

    const float delta = hd.delta;
    const float neg_off = -(float)(1 << (p.bits - 1)) * delta;  // exact: power of two times delta
    const int G = p.G;
    const uint32_t n_tiles = (n_chunks + G - 1) / G;

    for (uint32_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        // ---- variable length decoding into the LDS tile ----
        for (int j = wave; j < G; j += 4) {
            const uint32_t ch = tile * G + j;
            if (ch >= n_chunks) break;
            const uint64_t c0 = (uint64_t)ch * chunk_syms;
            const uint32_t clen = (uint32_t)((V - c0 < chunk_syms) ? (V - c0) : chunk_syms);
            // chunk bounds are the same for all lanes: keep them in scalar registers
            uint32_t w0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)chunk_off[ch]);
            uint32_t w1 = (uint32_t)__builtin_amdgcn_readfirstlane((int)chunk_off[ch + 1]);
            if (w0 > w1 || w1 > payload_words) {
                if (lane == 0) atomicOr(p.err, FMTC_ERR_OFFSETS);
                w0 = 0; w1 = 0;
            }
            const uint32_t run_bits = ((uint32_t)lane < spc) ? sub_bits[(size_t)ch * spc + lane] : 0u;
            const uint32_t start = dec_wave_exclusive_scan(run_bits, lane);
            const uint32_t r0 = (uint32_t)lane * kSubSyms;
            const uint32_t cnt = (r0 < clen) ? ((clen - r0 < (uint32_t)kSubSyms) ? clen - r0 : (uint32_t)kSubSyms) : 0u;
            const uint32_t nwords = w1 - w0;
            const uint32_t nbase = (uint32_t)j * chunk_syms + r0;
            uint32_t* pw = pay[wave];
            bool ok_run = true;
            if (nwords <= (uint32_t)kPayWords) {
                // the chunk's payload goes to LDS with full-width loads
                for (uint32_t i = lane; i < nwords + 2; i += 64) pw[i] = (i < nwords) ? payload[w0 + i] : 0u;
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                __builtin_amdgcn_wave_barrier();
                if (cnt)
                    ok_run = decode_run<true, ALIGNED4>(pw, nullptr, nwords, start, cnt, nbase, lut, cnt_len,
                                                        first_rank, first_code, sorted_sym, symtile);
                // the next chunk of this wavefront overwrites pay[]: all lanes are done reading here
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                __builtin_amdgcn_wave_barrier();
            } else if (cnt) {
                // a chunk too large for the LDS copy is read in place
                ok_run = decode_run<false, ALIGNED4>(nullptr, payload + w0, nwords, start, cnt, nbase, lut, cnt_len,
                                                     first_rank, first_code, sorted_sym, symtile);
            }
            if (!ok_run) atomicOr(p.err, FMTC_ERR_CODE);
        }
        __syncthreads();

        const uint32_t first_ch = tile * G;
        const uint32_t tile_chunks = (n_chunks - first_ch < (uint32_t)G) ? n_chunks - first_ch : (uint32_t)G;
        const uint64_t tile_s0 = (uint64_t)first_ch * chunk_syms;
        const uint32_t tile_syms = (uint32_t)((V - tile_s0 < (uint64_t)tile_chunks * chunk_syms)
                                                  ? (V - tile_s0) : (uint64_t)tile_chunks * chunk_syms);

        if (p.syms_out) {
            if constexpr (ALIGNED4) {
                for (uint32_t n = 4 * tid; n < tile_syms; n += 1024)
                    *reinterpret_cast<uint32_t*>(p.syms_out + tile_s0 + n) =
                        *reinterpret_cast<const uint32_t*>(symtile + sym_addr(n));
            } else {
                for (uint32_t n = tid; n < tile_syms; n += 256) p.syms_out[tile_s0 + n] = symtile[sym_addr(n)];
            }
        } else {
            // ---- inverse quantizer + inverse transform ----
            const int64_t px_tile0 = (int64_t)first_ch * (int64_t)ppc;
            const int TP = (int)(tile_syms / (uint32_t)C);  // pixels in this tile
            const int npt = (TP + 31) / 32;
            const int nptg = (npt + MT - 1) / MT;
            const int ct0 = blockIdx.y * p.ct_per_group;
            const int nct_g = (p.ncs - ct0 < p.ct_per_group) ? p.ncs - ct0 : p.ct_per_group;
            const int nunits = nct_g * nptg;
            for (int u = wave; u < nunits; u += 4) {
                const int ct = ct0 + u % nct_g;
                const int pt0 = (u / nct_g) * MT;
                uint32_t rowbase[MT];
#pragma unroll
                for (int m = 0; m < MT; m++) {
                    int pxl = (pt0 + m) * 32 + l32;
                    if (pxl > TP - 1) pxl = TP - 1;  // rows past the tile repeat the last pixel; never stored
                    rowbase[m] = (uint32_t)pxl * (uint32_t)C + 4u * half;
                }
                floatx16 acc[MT];
#pragma unroll
                for (int m = 0; m < MT; m++)
#pragma unroll
                    for (int r = 0; r < 16; r++) acc[m][r] = 0.f;

                const float4* bsrc = reinterpret_cast<const float4*>(p.Bpk + ((size_t)ct * p.ncs * 64 + lane) * 16);
                float4 b_cur[4], b_nxt[4];
#pragma unroll
                for (int q = 0; q < 4; q++) b_cur[q] = bsrc[q];
                for (int ks = 0; ks < p.ncs; ks++) {
                    if (ks + 1 < p.ncs) {
                        const float4* nsrc = bsrc + (size_t)(ks + 1) * 64 * 4;
#pragma unroll
                        for (int q = 0; q < 4; q++) b_nxt[q] = nsrc[q];
                    }
#pragma unroll
                    for (int t = 0; t < 4; t++) {
                        const float4 bv = b_cur[t];
                        const float bs[4] = {bv.x, bv.y, bv.z, bv.w};
#pragma unroll
                        for (int m = 0; m < MT; m++) {
                            const uint32_t n = rowbase[m] + (uint32_t)(ks * 32 + 8 * t);
                            uint32_t w;
                            if constexpr (ALIGNED4) {
                                w = *reinterpret_cast<const uint32_t*>(symtile + sym_addr(n));
                            } else {
                                w = (uint32_t)symtile[sym_addr(n)] | ((uint32_t)symtile[sym_addr(n + 1)] << 8) |
                                    ((uint32_t)symtile[sym_addr(n + 2)] << 16) | ((uint32_t)symtile[sym_addr(n + 3)] << 24);
                            }
#pragma unroll
                            for (int i = 0; i < 4; i++) {
                                float yq = __builtin_fmaf((float)((w >> (8 * i)) & 255u), delta, neg_off);
                                if constexpr (LAYOUT == FMTC_NHWC)
                                    acc[m] = __builtin_amdgcn_mfma_f32_32x32x2f32(yq, bs[i], acc[m], 0, 0, 0);
                                else
                                    acc[m] = __builtin_amdgcn_mfma_f32_32x32x2f32(bs[i], yq, acc[m], 0, 0, 0);
                            }
                        }
                    }
#pragma unroll
                    for (int q = 0; q < 4; q++) b_cur[q] = b_nxt[q];
                }

                // accumulator r of lane l is element (8*(r/4) + 4*(l/32) + r%4, l%32) of the 32x32 tile
                if constexpr (LAYOUT == FMTC_NHWC) {
                    const int c = ct * 32 + l32;
                    if (c < C) {
                        const float m_c = p.mu[c];
#pragma unroll
                        for (int m = 0; m < MT; m++)
#pragma unroll
                            for (int r = 0; r < 16; r++) {
                                int pxl = (pt0 + m) * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
                                if (pxl < TP) p.xhat[(px_tile0 + pxl) * C + c] = acc[m][r] + m_c;
                            }
                    }
                } else {
#pragma unroll
                    for (int m = 0; m < MT; m++) {
                        int pxl = (pt0 + m) * 32 + l32;
                        if (pxl < TP) {
                            int64_t px = px_tile0 + pxl;
                            int64_t n = px / p.HW, hw = px - n * p.HW;
                            float* dst = p.xhat + n * (int64_t)C * p.HW + hw;
#pragma unroll
                            for (int r = 0; r < 16; r++) {
                                int c = ct * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
                                if (c < C) dst[(int64_t)c * p.HW] = acc[m][r] + p.mu[c];
                            }
                        }
                    }
                }
            }
        }
        __syncthreads();
    }
}

hipError_t launch_decode(const BasisDevice* b, const uint8_t* d_stream, size_t bytes, const Geometry& g, int bits,
                         int64_t HW, int layout, float* d_xhat, uint8_t* d_syms, uint32_t* d_err, hipStream_t s) {
    const int C = g.C;
    const int ncs = (C + 31) / 32;
    // tile: enough chunks for at least 64 pixels at the nominal chunk size, 4..16 chunks
    int G = (int)((64 * (int64_t)C + 4095) / 4096);
    G = G < 4 ? 4 : (G > 16 ? 16 : (G + 3) / 4 * 4);
    DecodeParams p;
    p.stream = d_stream;
    p.bytes = bytes;
    p.P = g.P;
    p.HW = HW;
    p.C = C;
    p.bits = bits;
    p.G = G;
    p.ncs = ncs;
    p.Bpk = b ? b->inv : nullptr;
    p.mu = b ? b->mu : nullptr;
    p.xhat = d_xhat;
    p.syms_out = d_syms;
    p.err = d_err;
    // the grid is sized from the nominal geometry; the kernel takes the real one from the header
    const uint32_t n_tiles = (g.n_chunks + G - 1) / G;
    int groups = 1;
    if (!d_syms) {
        groups = (int)((256 + n_tiles - 1) / n_tiles);
        if (groups > ncs) groups = ncs;
        if (groups < 1) groups = 1;
    }
    p.ct_per_group = (ncs + groups - 1) / groups;
    groups = (ncs + p.ct_per_group - 1) / p.ct_per_group;
    unsigned gx = n_tiles < 2048u ? n_tiles : 2048u;
    dim3 grid(gx, (unsigned)groups);
    const size_t lds = (size_t)G * 4096 + (size_t)G * 4096 / 16 + 128;
    const bool al = (C % 4) == 0;
    ProfScope prof(K_DECODE, s);
    const bool wide = C > 256;  // fewer pixels per tile: 2 pixel tiles per wavefront unit instead of 4
    // more than 64 KB of dynamic LDS has to be requested per kernel (the CU has 160 KB)
#define FMTC_DEC(MT, LAY, AL)                                                                                \
    do {                                                                                                     \
        if (lds > 48 * 1024) {                                                                               \
            hipError_t ea = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_decode<MT, LAY, AL>),       \
                                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);      \
            if (ea != hipSuccess) return ea;                                                                 \
        }                                                                                                    \
        hipLaunchKernelGGL((k_decode<MT, LAY, AL>), grid, dim3(256), lds, s, p);                             \
    } while (0)
    if (layout == FMTC_NHWC) {
        if (al) { if (wide) FMTC_DEC(2, FMTC_NHWC, true); else FMTC_DEC(4, FMTC_NHWC, true); }
        else    { if (wide) FMTC_DEC(2, FMTC_NHWC, false); else FMTC_DEC(4, FMTC_NHWC, false); }
    } else {
        if (al) { if (wide) FMTC_DEC(2, FMTC_NCHW, true); else FMTC_DEC(4, FMTC_NCHW, true); }
        else    { if (wide) FMTC_DEC(2, FMTC_NCHW, false); else FMTC_DEC(4, FMTC_NCHW, false); }
    }
#undef FMTC_DEC
    return hipGetLastError();
}

}  // namespace fmtc
