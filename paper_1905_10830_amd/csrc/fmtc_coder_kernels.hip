// Variable length coder (paper section 3.1 "Variable length coding"; appendix
// "Huffman encoder as VLC"): Huffman code lengths from the symbol histogram,
// canonical code words, per-run bit counts, chunk offsets and the packed stream.
// All integer work; results are unique, so they are bit-exact by construction.
#include "fmtc_internal.h"

namespace fmtc {

// ---------------------------------------------------------------------------
// Code table.  One workgroup.  Lengths follow the classic construction: leaves
// ordered by (count, symbol), the two lightest nodes merged until one is left; a
// leaf wins over an internal node of equal weight, internal nodes leave in the
// order they were made.  Codes are canonical in (length, symbol) order.
// ---------------------------------------------------------------------------
// one value of a per-lane array spread over NV registers (64 entries each); idx is wavefront-uniform
template <int NV>
__device__ __forceinline__ uint32_t lane_get(const uint32_t (&v)[NV], int idx) {
    uint32_t r = (uint32_t)__builtin_amdgcn_readlane((int)v[0], idx & 63);
#pragma unroll
    for (int j = 1; j < NV; j++) {
        uint32_t t = (uint32_t)__builtin_amdgcn_readlane((int)v[j], idx & 63);
        r = ((idx >> 6) == j) ? t : r;
    }
    return r;
}
template <int NV>
__device__ __forceinline__ void lane_set(uint32_t (&v)[NV], int lane, int idx, uint32_t val) {
#pragma unroll
    for (int j = 0; j < NV; j++) v[j] = (64 * j + lane == idx) ? val : v[j];
}

// The merge loop is serial by nature (n-1 steps).  It runs in one wavefront with
// the two queues held in registers across the lanes and all control in scalar
// registers, so a step costs a few lane reads/writes instead of LDS round trips.
// NV * 64 >= alphabet size.
template <int NV>
__global__ __launch_bounds__(1024) void k_huffman_table(const uint32_t* __restrict__ hist_parts, int n_parts,
                                                        int bits, uint32_t* __restrict__ hist_out,
                                                        uint64_t* __restrict__ enc_table,
                                                        uint8_t* __restrict__ len_table,
                                                        uint32_t* __restrict__ counters) {
    __shared__ uint32_t h[256];
    __shared__ uint32_t weight[256];       // leaf weights in (count, symbol) order
    __shared__ uint16_t leaf_parent[256];  // index of the internal node above each sorted leaf
    __shared__ uint16_t int_parent[256];   // ... above each internal node (creation order)
    __shared__ uint8_t len[256];
    __shared__ uint32_t len_count[kMaxLen + 2];
    __shared__ uint64_t first_code[kMaxLen + 2];
    __shared__ int n_used;

    const int s = threadIdx.x;
    const int K = 1 << bits;
    if (s < 256) {
        h[s] = 0u;
        len[s] = 0;
    }
    if (s <= kMaxLen + 1) len_count[s] = 0;
    if (s == 0) n_used = 0;
    if (s < 16) counters[s] = 0u;  // tickets of the kernels that follow in this call
    __syncthreads();
    {
        // sum of the partial histograms: 1024 / K threads share a bin
        const int bin = s & (K - 1), first = s >> bits, step = 1024 >> bits;
        uint32_t part = 0;
        int q = first;
        for (; q + 7 * step < n_parts; q += 8 * step) {  // eight independent loads in flight
            uint32_t v[8];
#pragma unroll
            for (int j = 0; j < 8; j++) v[j] = hist_parts[(size_t)(q + j * step) * K + bin];
#pragma unroll
            for (int j = 0; j < 8; j++) part += v[j];
        }
        for (; q < n_parts; q += step) part += hist_parts[(size_t)q * K + bin];
        if (part) atomicAdd(&h[bin], part);
    }
    __syncthreads();
    // from here on at most one thread per symbol works; the others only keep the barriers company
    const uint32_t cnt = s < 256 ? h[s] : 0u;
    if (s < 256) hist_out[s] = cnt;

    // rank of every used symbol in (count, symbol) order
    int rank = 0;
    if (cnt) {
        for (int t = 0; t < K; t++) {
            uint32_t o = h[t];
            rank += (o != 0 && (o < cnt || (o == cnt && t < s))) ? 1 : 0;
        }
        weight[rank] = cnt;
        atomicAdd(&n_used, 1);
    }
    __syncthreads();
    const int n = __builtin_amdgcn_readfirstlane(n_used);

    if (s < 64 && n >= 2) {
        const int lane = s;
        uint32_t lw[NV], iw[NV], lpar[NV], ipar[NV];
#pragma unroll
        for (int j = 0; j < NV; j++) {
            lw[j] = (64 * j + lane < n) ? weight[64 * j + lane] : 0xffffffffu;
            iw[j] = 0xffffffffu;
            lpar[j] = 0;
            ipar[j] = 0;
        }
        // an exhausted queue shows weight 2^32-1; no node that can still be picked weighs that much (V < 2^32)
        int nl = 0, ni = 0, made = 0;
        uint32_t lh = lane_get<NV>(lw, 0), ih = 0xffffffffu;
        for (int m = 0; m < n - 1; m++) {
            uint32_t w = 0;
#pragma unroll
            for (int t = 0; t < 2; t++) {
                if (lh <= ih) {  // a leaf wins over an internal node of equal weight
                    w += lh;
                    lane_set<NV>(lpar, lane, nl, (uint32_t)made);
                    nl++;
                    lh = (nl < n) ? lane_get<NV>(lw, nl) : 0xffffffffu;
                } else {
                    w += ih;
                    lane_set<NV>(ipar, lane, ni, (uint32_t)made);
                    ni++;
                    ih = (ni < made) ? lane_get<NV>(iw, ni) : 0xffffffffu;
                }
            }
            lane_set<NV>(iw, lane, made, w);
            if (ni == made) ih = w;  // the new node heads an empty internal queue
            made++;
        }
#pragma unroll
        for (int j = 0; j < NV; j++) {
            leaf_parent[64 * j + lane] = (uint16_t)lpar[j];
            int_parent[64 * j + lane] = (uint16_t)ipar[j];
        }
    }
    __syncthreads();

    if (cnt) {
        int l = 1;
        if (n >= 2) {
            const int root = n - 2;
            int cur = leaf_parent[rank];
            while (cur != root && l <= kMaxLen) {  // depth = number of ancestors
                cur = int_parent[cur];
                l++;
            }
        }
        if (l > kMaxLen) l = kMaxLen;  // unreachable for V < 2^32 (depth d needs a total count >= Fibonacci(d+2))
        len[s] = (uint8_t)l;
        atomicAdd(&len_count[l], 1u);
    }
    __syncthreads();
    if (s >= 1 && s <= kMaxLen) {
        // first canonical code of every length: code(l) = sum_{j<l} count(j) << (l-j)
        uint64_t code = 0;
        for (int j = 1; j < s; j++) code += (uint64_t)len_count[j] << (s - j);
        first_code[s] = code;
    }
    __syncthreads();
    if (s < 256) {
        const int l = len[s];
        uint64_t entry = 0;
        if (l) {
            int before = 0;
            for (int t = 0; t < s; t++) before += (len[t] == l) ? 1 : 0;
            uint64_t code = first_code[l] + (uint64_t)before;
            uint64_t rev = __brevll(code) >> (64 - l);  // stream order is least significant bit first
            entry = rev | ((uint64_t)l << 56);
        }
        enc_table[s] = entry;
        len_table[s] = (uint8_t)l;
    }
}

hipError_t launch_huffman_table(const uint32_t* d_hist_parts, int n_parts, int bits, uint32_t* d_hist,
                                uint64_t* d_enc_table, uint8_t* d_len_table, uint32_t* d_counters, hipStream_t s) {
    ProfScope prof(K_TABLE, s);
    if (bits <= 6)
        hipLaunchKernelGGL(k_huffman_table<1>, dim3(1), dim3(1024), 0, s, d_hist_parts, n_parts, bits, d_hist,
                           d_enc_table, d_len_table, d_counters);
    else if (bits == 7)
        hipLaunchKernelGGL(k_huffman_table<2>, dim3(1), dim3(1024), 0, s, d_hist_parts, n_parts, bits, d_hist,
                           d_enc_table, d_len_table, d_counters);
    else
        hipLaunchKernelGGL(k_huffman_table<4>, dim3(1), dim3(1024), 0, s, d_hist_parts, n_parts, bits, d_hist,
                           d_enc_table, d_len_table, d_counters);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Pass 1 of packing: code bits of every run of 64 symbols and of every chunk.
// One wavefront per chunk, one lane per run.
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// exclusive prefix sum over the 64 lanes
__device__ __forceinline__ uint32_t wave_exclusive_scan(uint32_t v, int lane) {
    uint32_t incl = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        uint32_t t = __shfl_up(incl, o, 64);
        if (lane >= o) incl += t;
    }
    return incl - v;
}

// The last workgroup to finish (ticket counter, reset by the table kernel) turns the chunk sizes into
// offsets: exclusive scan in words, header, stream size.  Every thread of it owns a contiguous segment.
__global__ __launch_bounds__(256) void k_run_bits(const uint8_t* __restrict__ syms, uint64_t V, uint32_t n_chunks,
                                                  uint32_t chunk_syms, uint32_t subs_per_chunk,
                                                  const uint64_t* __restrict__ enc_table,
                                                  uint16_t* __restrict__ sub_bits, uint32_t* chunk_bits,
                                                  uint32_t* ticket, Header hdr, size_t off_sub_bits,
                                                  size_t off_payload, uint8_t* __restrict__ stream,
                                                  uint64_t* __restrict__ out_bytes) {
    __shared__ uint8_t llen[256];
    __shared__ uint32_t wave_words[4];
    __shared__ unsigned long long wave_bits[4];
    __shared__ uint32_t is_last;
    llen[threadIdx.x] = (uint8_t)(enc_table[threadIdx.x] >> 56);
    __syncthreads();
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t ch = blockIdx.x * 4 + (uint32_t)wave;
    if (ch < n_chunks) {
        const uint64_t c0 = (uint64_t)ch * chunk_syms;
        const uint64_t c1 = (c0 + chunk_syms < V) ? c0 + chunk_syms : V;
        const uint64_t r0 = c0 + (uint64_t)lane * kSubSyms;
        uint32_t bits = 0;
        if (r0 < c1) {
            const uint32_t cnt = (uint32_t)((c1 - r0 < kSubSyms) ? (c1 - r0) : kSubSyms);
            if (cnt == kSubSyms && ((uintptr_t)(syms + r0) & 15) == 0) {
                const uint4* p = reinterpret_cast<const uint4*>(syms + r0);
#pragma unroll
                for (int j = 0; j < 4; j++) {
                    uint4 v = p[j];
                    uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                    for (int q = 0; q < 4; q++)
#pragma unroll
                        for (int b = 0; b < 4; b++) bits += llen[(w[q] >> (8 * b)) & 255];
                }
            } else {
                for (uint32_t i = 0; i < cnt; i++) bits += llen[syms[r0 + i]];
            }
        }
        if ((uint32_t)lane < subs_per_chunk) sub_bits[(size_t)ch * subs_per_chunk + lane] = (uint16_t)bits;
        uint32_t total = wave_sum(bits);
        if (lane == 0) chunk_bits[ch] = total;
    }
    // ---- ticket: has every other workgroup published its chunk sizes? ----
    // one release per workgroup (a cache write-back on this chip), not one per wavefront
    __syncthreads();
    if (tid == 0) {
        __threadfence();
        is_last = (atomicAdd(ticket, 1u) == gridDim.x - 1) ? 1u : 0u;
    }
    __syncthreads();
    if (!is_last) return;
    __threadfence();

    uint32_t* chunk_off = reinterpret_cast<uint32_t*>(stream + kHeaderBytes + kLenTableBytes);
    const uint32_t seg = (n_chunks + 255) / 256;
    const uint32_t i0 = (uint32_t)tid * seg;
    const uint32_t i1 = (i0 + seg < n_chunks) ? i0 + seg : n_chunks;
    uint32_t words = 0;
    unsigned long long nbits = 0;
    for (uint32_t i = i0; i < i1; i++) {
        uint32_t b = __atomic_load_n(&chunk_bits[i], __ATOMIC_RELAXED);
        words += (b + 31) >> 5;
        nbits += b;
    }
    uint32_t ex = wave_exclusive_scan(words, lane);
    unsigned long long bsum = nbits;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) bsum += __shfl_xor(bsum, o, 64);
    if (lane == 63) wave_words[wave] = ex + words;
    if (lane == 0) wave_bits[wave] = bsum;
    __syncthreads();
    uint32_t base = ex;
    for (int q = 0; q < wave; q++) base += wave_words[q];
    for (uint32_t i = i0; i < i1; i++) {
        chunk_off[i] = base;
        base += (__atomic_load_n(&chunk_bits[i], __ATOMIC_RELAXED) + 31) >> 5;
    }
    if (tid == 0) {
        uint64_t total_words = 0, total_bits = 0;
        for (int q = 0; q < 4; q++) {
            total_words += wave_words[q];
            total_bits += wave_bits[q];
        }
        chunk_off[n_chunks] = (uint32_t)total_words;
        hdr.payload_words = total_words;
        hdr.payload_bits = total_bits;
        *reinterpret_cast<Header*>(stream) = hdr;
        if (out_bytes) *out_bytes = (uint64_t)off_payload + 4 * total_words;
        // alignment gaps between the sections are part of the stream: keep them zero
        for (size_t o = kHeaderBytes + kLenTableBytes + 4 * ((size_t)n_chunks + 1); o < off_sub_bits; o++) stream[o] = 0;
        for (size_t o = off_sub_bits + 2 * (size_t)n_chunks * hdr.subs_per_chunk; o < off_payload; o++) stream[o] = 0;
    }
}

// ---------------------------------------------------------------------------
// Pass 2 of packing.  One wavefront per chunk, one lane per run.  The lane's
// bit offset inside the chunk is the prefix sum of the run sizes; codes are
// appended least significant stream bit first into a 64-bit register and
// leave as 32-bit words OR-ed into an LDS image of the chunk, which is then
// copied out with full-width stores.  A chunk larger than the LDS image is
// produced in several windows (the runs are re-read per window).
// ---------------------------------------------------------------------------
constexpr int kStageWords = 2048;  // per wavefront: 64 Kbit, i.e. 16 bits/symbol over a 4096-symbol chunk

__global__ __launch_bounds__(256) void k_pack(const uint8_t* __restrict__ syms, uint64_t V, uint32_t n_chunks,
                                              uint32_t chunk_syms, uint32_t subs_per_chunk,
                                              const uint64_t* __restrict__ enc_table,
                                              const uint16_t* __restrict__ sub_bits,
                                              const uint32_t* __restrict__ chunk_off,
                                              uint32_t* __restrict__ payload) {
    __shared__ uint64_t tab[256];
    __shared__ uint32_t stage[4][kStageWords];
    tab[threadIdx.x] = enc_table[threadIdx.x];
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));  // wavefront-uniform by construction
    const uint32_t ch = blockIdx.x * 4 + wave;
    if (ch >= n_chunks) return;  // whole wavefront leaves; no workgroup barrier follows
    uint32_t* img = stage[wave];
    const uint64_t c0 = (uint64_t)ch * chunk_syms;
    const uint64_t c1 = (c0 + chunk_syms < V) ? c0 + chunk_syms : V;
    const uint64_t r0 = c0 + (uint64_t)lane * kSubSyms;
    const uint32_t cnt = (r0 < c1) ? (uint32_t)((c1 - r0 < kSubSyms) ? (c1 - r0) : kSubSyms) : 0u;
    const uint32_t my_bits = ((uint32_t)lane < subs_per_chunk) ? sub_bits[(size_t)ch * subs_per_chunk + lane] : 0u;
    const uint32_t start = wave_exclusive_scan(my_bits, lane);
    const uint32_t total_bits = __shfl(start + my_bits, 63, 64);
    const uint32_t n_words = (total_bits + 31) >> 5;
    uint32_t* out = payload + (uint32_t)__builtin_amdgcn_readfirstlane((int)chunk_off[ch]);

    for (uint32_t win = 0; win < n_words; win += kStageWords) {
        const uint32_t win_words = (n_words - win < (uint32_t)kStageWords) ? n_words - win : (uint32_t)kStageWords;
        for (uint32_t i = lane; i < win_words; i += 64) img[i] = 0u;
        // LDS operations of one wavefront complete in order: the zeros land before the ORs below
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        const uint32_t first_word = start >> 5, last_word = (start + my_bits + 31) >> 5;  // [first, last)
        if (cnt && my_bits && first_word < win + win_words && last_word > win) {
            uint64_t acc = 0;
            uint32_t nb = start & 31;
            uint32_t widx = first_word;
            auto emit = [&](uint32_t word) {
                uint32_t rel = widx - win;
                if (rel < win_words) atomicOr(&img[rel], word);
                widx++;
            };
            auto put = [&](uint64_t code, uint32_t len) {  // len <= 32, nb < 32
                acc |= code << nb;
                nb += len;
                if (nb >= 32) {
                    emit((uint32_t)acc);
                    acc >>= 32;
                    nb -= 32;
                }
            };
            auto code_symbol = [&](uint32_t sym) {
                uint64_t e = tab[sym];
                uint32_t len = (uint32_t)(e >> 56);
                uint64_t code = e & 0x00ffffffffffffffull;
                if (len > 32) {
                    put(code & 0xffffffffull, 32);
                    put(code >> 32, len - 32);
                } else {
                    put(code, len);
                }
            };
            if (cnt == kSubSyms && ((uintptr_t)(syms + r0) & 15) == 0) {
                const uint4* p = reinterpret_cast<const uint4*>(syms + r0);
#pragma unroll
                for (int j = 0; j < 4; j++) {
                    uint4 v = p[j];
                    uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                    for (int q = 0; q < 4; q++)
#pragma unroll
                        for (int b = 0; b < 4; b++) code_symbol((w[q] >> (8 * b)) & 255);
                }
            } else {
                for (uint32_t i = 0; i < cnt; i++) code_symbol(syms[r0 + i]);
            }
            if (nb) emit((uint32_t)acc);
        }
        // the ORs of all lanes precede the reads below: one wavefront, LDS in order
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        for (uint32_t i = lane; i < win_words; i += 64) out[win + i] = img[i];
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}

hipError_t launch_pack(const uint8_t* d_syms, const Geometry& g, int bits, float delta, const uint64_t* d_enc_table,
                       uint32_t* d_chunk_bits, uint32_t* d_counters, uint8_t* d_stream, uint64_t* d_out_bytes,
                       hipStream_t s) {
    const uint64_t V = (uint64_t)g.P * (uint64_t)g.C;
    uint16_t* sub_bits = reinterpret_cast<uint16_t*>(d_stream + g.off_sub_bits);
    uint32_t* chunk_off = reinterpret_cast<uint32_t*>(d_stream + g.off_chunk_off);
    uint32_t* payload = reinterpret_cast<uint32_t*>(d_stream + g.off_payload);
    const unsigned blocks = (g.n_chunks + 3) / 4;
    Header hdr = {};
    hdr.magic = kMagic;
    hdr.version = 1;
    hdr.bits = (uint8_t)bits;
    hdr.C = (uint32_t)g.C;
    hdr.px_per_chunk = g.px_per_chunk;
    hdr.P = (uint64_t)g.P;
    hdr.n_chunks = g.n_chunks;
    hdr.sub_syms = kSubSyms;
    hdr.delta = delta;
    hdr.subs_per_chunk = g.subs_per_chunk;
    {
        ProfScope prof(K_RUN_BITS, s);
        hipLaunchKernelGGL(k_run_bits, dim3(blocks), dim3(256), 0, s, d_syms, V, g.n_chunks, g.chunk_syms,
                           g.subs_per_chunk, d_enc_table, sub_bits, d_chunk_bits, d_counters + 1, hdr, g.off_sub_bits,
                           g.off_payload, d_stream, d_out_bytes);
    }
    {
        ProfScope prof(K_PACK, s);
        hipLaunchKernelGGL(k_pack, dim3(blocks), dim3(256), 0, s, d_syms, V, g.n_chunks, g.chunk_syms,
                           g.subs_per_chunk, d_enc_table, sub_bits, chunk_off, payload);
    }
    return hipGetLastError();
}

}  // namespace fmtc
