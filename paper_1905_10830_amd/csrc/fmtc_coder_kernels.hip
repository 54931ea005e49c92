// Variable length coder (paper section 3.1 "Variable length coding"; appendix
// "Huffman encoder as VLC"): Huffman code lengths from the symbol histogram,
// canonical code words, per-run bit counts, chunk offsets and the packed stream.
// All integer work; results are unique, so they are bit-exact by construction.
//
// Two kernels at most:
//   k_huffman_table  one workgroup: sums the partial histograms and builds the code
//                    (large tensors; small ones build it inside the pack kernel, every
//                    workgroup for itself, which saves a launch on the critical path);
//   k_pack           one wavefront per chunk, one lane per run of 64 symbols: run sizes,
//                    the chunk's place in the payload (a running sum over the chunk
//                    groups handed from workgroup to workgroup), then the code bits.
#include <cstdlib>

#include "fmtc_device.h"
#include "fmtc_internal.h"

namespace fmtc {

constexpr uint32_t kInf = 0xffffffffu;

// ---------------------------------------------------------------------------
// Code table.  Lengths follow the classic construction: leaves ordered by
// (count, symbol), the two lightest nodes merged until one is left; a leaf wins
// over an internal node of equal weight, internal nodes leave in the order they
// were made.  Codes are canonical in (length, symbol) order.
// ---------------------------------------------------------------------------
struct TableLds {
    uint32_t h[256];
    uint32_t weight[256];       // leaf weights in (count, symbol) order
    uint32_t rank[256];         // position of every used symbol in that order
    uint32_t children[256];     // per merge: node ids of the two children (leaf i: i, internal j: 256 + j)
    uint16_t leaf_parent[256];  // merge that consumed each sorted leaf
    uint16_t int_parent[256];   // ... each internal node (numbered in creation order)
    uint8_t len[256];
    uint32_t len_count[64];
    uint32_t wave_len_count[4][64];
    unsigned long long first_code[64];
    unsigned long long entry[256];  // result: bit-reversed code | length << 56
    unsigned long long payload_bits;
    uint32_t n_used, max_len;
};

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
__device__ __forceinline__ void lane_put(uint32_t (&v)[NV], int lane, int idx, uint32_t val) {
#pragma unroll
    for (int j = 0; j < NV; j++) v[j] = (64 * j + lane == idx) ? val : v[j];
}

// The merge loop is serial by nature (n-1 steps).  It runs in one wavefront with the two queues held in
// registers across the lanes and all control in scalar registers.  NV * 64 >= number of used symbols.
template <int NV>
__device__ __forceinline__ void huffman_merge(TableLds& L, int lane, int n) {
    uint32_t lw[NV], iw[NV], ch[NV];
#pragma unroll
    for (int j = 0; j < NV; j++) {
        lw[j] = (64 * j + lane < n) ? L.weight[64 * j + lane] : kInf;
        iw[j] = kInf;  // nodes not made yet weigh "infinity"; no node that can still be picked does (V < 2^32)
        ch[j] = 0;
    }
    int nl = 0, ni = 0;
    for (int made = 0; made < n - 1; made++) {
        const uint32_t l0 = (nl < n) ? lane_get<NV>(lw, nl) : kInf;
        const uint32_t l1 = (nl + 1 < n) ? lane_get<NV>(lw, nl + 1) : kInf;
        const uint32_t i0 = (ni < made) ? lane_get<NV>(iw, ni) : kInf;
        const uint32_t i1 = (ni + 1 < made) ? lane_get<NV>(iw, ni + 1) : kInf;
        // first pick: a leaf wins over an internal node of equal weight
        const bool a_leaf = l0 <= i0;
        const uint32_t wa = a_leaf ? l0 : i0;
        const uint32_t ida = a_leaf ? (uint32_t)nl : 256u + (uint32_t)ni;
        const uint32_t ln = a_leaf ? l1 : l0, in = a_leaf ? i0 : i1;
        const int nl1 = nl + (a_leaf ? 1 : 0), ni1 = ni + (a_leaf ? 0 : 1);
        const bool b_leaf = ln <= in;
        const uint32_t wb = b_leaf ? ln : in;
        const uint32_t idb = b_leaf ? (uint32_t)nl1 : 256u + (uint32_t)ni1;
        nl = nl1 + (b_leaf ? 1 : 0);
        ni = ni1 + (b_leaf ? 0 : 1);
        lane_put<NV>(iw, lane, made, wa + wb);
        lane_put<NV>(ch, lane, made, ida | (idb << 16));
    }
#pragma unroll
    for (int j = 0; j < NV; j++) L.children[64 * j + lane] = ch[j];
}

// Builds the table from the partial histograms into L.  All THREADS threads of the workgroup call it.
// THREADS is a multiple of 256.
template <int THREADS>
__device__ __forceinline__ void build_table(TableLds& L, const uint32_t* __restrict__ hist_parts, int n_parts,
                                            int bits) {
    const int tid = threadIdx.x, lane = tid & 63;
    const int K = 1 << bits;
    if (tid < 256) {
        L.h[tid] = 0u;
        L.rank[tid] = 0u;
        L.len[tid] = 0;
        L.wave_len_count[tid >> 6][tid & 63] = 0u;
    }
    if (tid < 64) L.len_count[tid] = 0u;
    if (tid == 0) {
        L.n_used = 0u;
        L.payload_bits = 0ull;
        L.max_len = 0u;
    }
    __syncthreads();
    {
        // sum of the partial histograms: THREADS / K threads share a bin, eight independent loads in flight
        const int bin = tid & (K - 1), first = tid >> bits, step = THREADS >> bits;
        uint32_t part = 0;
        int q = first;
        for (; q + 7 * step < n_parts; q += 8 * step) {
            uint32_t v[8];
#pragma unroll
            for (int j = 0; j < 8; j++) v[j] = hist_parts[(size_t)(q + j * step) * K + bin];
#pragma unroll
            for (int j = 0; j < 8; j++) part += v[j];
        }
        for (; q < n_parts; q += step) part += hist_parts[(size_t)q * K + bin];
        if (part) atomicAdd(&L.h[bin], part);
    }
    __syncthreads();
    // rank of every used symbol in (count, symbol) order: THREADS / 256 threads share a symbol
    const int s = tid & 255, part_id = tid >> 8;
    constexpr int kParts = THREADS / 256;
    const uint32_t cnt = L.h[s];
    if (cnt) {
        uint32_t r = 0;
        for (int t = part_id; t < K; t += kParts) {
            const uint32_t o = L.h[t];
            r += (o != 0 && (o < cnt || (o == cnt && t < s))) ? 1u : 0u;
        }
        if (r) atomicAdd(&L.rank[s], r);
        if (part_id == 0) atomicAdd(&L.n_used, 1u);
    }
    __syncthreads();
    const int n = __builtin_amdgcn_readfirstlane((int)L.n_used);
    const uint32_t rank = L.rank[s];
    if (cnt && part_id == 0) L.weight[rank] = cnt;
    __syncthreads();

    if (tid < 64 && n >= 2) {
        if (n <= 64) huffman_merge<1>(L, lane, n);
        else if (n <= 128) huffman_merge<2>(L, lane, n);
        else huffman_merge<4>(L, lane, n);
    }
    __syncthreads();
    if (tid < n - 1) {
        const uint32_t c = L.children[tid];
        const uint32_t a = c & 0xffffu, b = c >> 16;
        if (a < 256u) L.leaf_parent[a] = (uint16_t)tid; else L.int_parent[a - 256u] = (uint16_t)tid;
        if (b < 256u) L.leaf_parent[b] = (uint16_t)tid; else L.int_parent[b - 256u] = (uint16_t)tid;
    }
    __syncthreads();

    int l = 0;
    if (cnt && part_id == 0) {
        l = 1;
        if (n >= 2) {
            const int root = n - 2;
            int cur = L.leaf_parent[rank];
            while (cur != root && l <= kMaxLen) {  // depth = number of ancestors
                cur = L.int_parent[cur];
                l++;
            }
        }
        if (l > kMaxLen) l = kMaxLen;  // unreachable for V < 2^32 (depth d needs a total count >= Fibonacci(d+2))
        L.len[s] = (uint8_t)l;
        atomicAdd(&L.len_count[l], 1u);
        atomicAdd(&L.payload_bits, (unsigned long long)cnt * (unsigned long long)l);
    }
    __syncthreads();
    if (tid < 64) {
        // first canonical code of every length: code(l) = sum_{j<l} count(j) << (l-j), i.e. the running sum of
        // count(j) * 2^(48-j) shifted down to l bits
        const bool in = tid >= 1 && tid <= kMaxLen;
        const uint32_t c = in ? L.len_count[tid] : 0u;
        const unsigned long long w = (unsigned long long)c << (in ? kMaxLen - tid : 0);
        const unsigned long long incl = wave_inclusive_scan64(w, lane);
        L.first_code[tid] = in ? ((incl - w) >> (kMaxLen - tid)) : 0ull;
        const unsigned long long used = __ballot(c != 0);
        if (tid == 0) L.max_len = used ? (uint32_t)(63 - __clzll((long long)used)) : 0u;
    }
    __syncthreads();
    // symbols of equal length are numbered in symbol order: count those before this one
    uint32_t before = 0;
    if (tid < 256) {
        const uint32_t max_len = L.max_len;
        for (uint32_t q = 1; q <= max_len; q++) {
            const unsigned long long m = __ballot(l == (int)q);
            if (l == (int)q) before = (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
            if (lane == 0 && m) L.wave_len_count[tid >> 6][q] = (uint32_t)__popcll(m);
        }
    }
    __syncthreads();
    if (tid < 256) {
        unsigned long long entry = 0;
        if (l) {
            for (int q = 0; q < (tid >> 6); q++) before += L.wave_len_count[q][l];
            const unsigned long long code = L.first_code[l] + (unsigned long long)before;
            const unsigned long long rev = __brevll(code) >> (64 - l);  // stream order: least significant bit first
            entry = rev | ((unsigned long long)l << 56);
        }
        L.entry[tid] = entry;
    }
    __syncthreads();
}

__global__ __launch_bounds__(1024) void k_huffman_table(const uint32_t* __restrict__ hist_parts, int n_parts,
                                                        int bits, uint32_t* __restrict__ hist_out,
                                                        uint64_t* __restrict__ enc_table,
                                                        uint8_t* __restrict__ len_table,
                                                        CoderCtrl* __restrict__ ctrl) {
    __shared__ TableLds L;
    build_table<1024>(L, hist_parts, n_parts, bits);
    const int tid = threadIdx.x;
    if (tid < 256) {
        if (hist_out) hist_out[tid] = L.h[tid];
        if (enc_table) enc_table[tid] = L.entry[tid];
        if (len_table) len_table[tid] = L.len[tid];
    }
    if (tid == 0 && ctrl) {
        ctrl->max_len = L.max_len;
        ctrl->payload_bits = L.payload_bits;
    }
}

// Sum of the partial histograms only.
__global__ __launch_bounds__(256) void k_histogram_sum(const uint32_t* __restrict__ hist_parts, int n_parts,
                                                       int bits, uint32_t* __restrict__ hist_out) {
    const int K = 1 << bits, s = threadIdx.x;
    uint32_t acc = 0;
    if (s < K)
        for (int q = 0; q < n_parts; q++) acc += hist_parts[(size_t)q * K + s];
    hist_out[s] = acc;
}

hipError_t launch_histogram_sum(const uint32_t* d_hist_parts, int n_parts, int bits, uint32_t* d_hist,
                                hipStream_t s) {
    return launch(K_TABLE, k_histogram_sum, dim3(1), dim3(256), 0, s, d_hist_parts, n_parts, bits, d_hist);
}

// ---------------------------------------------------------------------------
// Packing.  One wavefront per chunk, one lane per run of 64 symbols, the run in
// registers.  Pass 1 sums the code lengths of the run; the prefix sum over the
// lanes gives each run's bit offset in the chunk.  The chunk's first payload
// word is the number of words of all chunks before it: workgroups take their
// chunk group from a ticket counter (so a group's predecessors are always
// running already), publish the group's word count, and read back over their
// predecessors' published counts until they meet one that is already a running
// total.  Pass 2 appends the codes, least significant stream bit first, into an
// LDS image of the chunk that leaves with full-width stores.  A chunk larger
// than the image is produced in several windows.
// ---------------------------------------------------------------------------
constexpr int kStageWords = 2048;  // per wavefront: 64 Kbit, i.e. 16 bits/symbol over a 4096-symbol chunk
constexpr unsigned long long kFlagAggregate = 1ull << 32, kFlagInclusive = 2ull << 32;
constexpr uint32_t kSpinLimit = 1u << 22;  // polls before a wait gives up (seconds; never reached unless the
                                           // workspace is overwritten while the kernel runs)

struct PackParams {
    const uint8_t* syms;
    uint64_t V;
    uint32_t n_chunks, chunk_syms, subs_per_chunk, n_groups;
    int bits;
    const uint32_t* hist_parts;  // BUILD: partial histograms to build the table from
    int n_parts;
    const uint64_t* enc_table;   // !BUILD: table made by k_huffman_table
    CoderCtrl* ctrl;
    unsigned long long* lookback;
    Header hdr;
    size_t off_sub_bits, off_payload;
    uint8_t* stream;
    uint64_t* out_bytes;
};

// Appends the codes of one run to the image.  FULL: the run has all 64 symbols.  LONG: codes may exceed 32 bits.
template <bool FULL, bool LONG>
__device__ __forceinline__ void pack_run(const uint32_t (&w)[16], uint32_t cnt, uint32_t start,
                                         const unsigned long long* tab, uint32_t* img, uint32_t win,
                                         uint32_t win_words) {
    uint32_t nb = start & 31, widx = start >> 5;
    auto emit = [&](uint32_t word) {
        const uint32_t rel = widx - win;
        if (rel < win_words) atomicOr(&img[rel], word);
        widx++;
    };
    if constexpr (!LONG) {
        uint32_t lo = 0;
#pragma unroll
        for (int q = 0; q < 16; q++)
#pragma unroll
            for (int b = 0; b < 4; b++) {
                if (FULL || (uint32_t)(4 * q + b) < cnt) {
                    const unsigned long long e = tab[(w[q] >> (8 * b)) & 255u];
                    const uint32_t code = (uint32_t)e, len = (uint32_t)(e >> 56);
                    lo |= code << nb;
                    const uint32_t hi = (code >> 1) >> (31 - nb);  // bits of the code that do not fit the word
                    nb += len;
                    if (nb >= 32) {
                        emit(lo);
                        lo = hi;
                        nb -= 32;
                    }
                }
            }
        if (nb) emit(lo);
    } else {
        unsigned long long acc = 0;
        auto put = [&](unsigned long long code, uint32_t len) {  // len <= 32, nb < 32
            acc |= code << nb;
            nb += len;
            if (nb >= 32) {
                emit((uint32_t)acc);
                acc >>= 32;
                nb -= 32;
            }
        };
#pragma unroll 1
        for (uint32_t i = 0; i < cnt; i++) {
            uint32_t word = 0;
#pragma unroll
            for (int q = 0; q < 16; q++) word = ((i >> 2) == (uint32_t)q) ? w[q] : word;
            const unsigned long long e = tab[(word >> (8 * (i & 3))) & 255u];
            const uint32_t len = (uint32_t)(e >> 56);
            const unsigned long long code = e & 0x00ffffffffffffffull;
            if (len > 32) {
                put(code & 0xffffffffull, 32);
                put(code >> 32, len - 32);
            } else {
                put(code, len);
            }
        }
        if (nb) emit((uint32_t)acc);
    }
}

template <bool BUILD>
__global__ __launch_bounds__(256) void k_pack(PackParams p) {
    __shared__ unsigned long long tab[256];
    __shared__ __align__(16) uint32_t stage[kPackWaves][kStageWords];
    __shared__ uint32_t wave_words[kPackWaves];
    __shared__ uint32_t s_group, s_excl, s_max_len;
    __shared__ unsigned long long s_payload_bits;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wavefront-uniform by construction
    if (tid == 0) s_group = __hip_atomic_fetch_add(&p.ctrl->ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if constexpr (BUILD) {
        // the table scratch shares LDS with the chunk images, which are not in use yet
        static_assert(sizeof(TableLds) <= sizeof(stage), "table scratch must fit the chunk images");
        TableLds& L = *reinterpret_cast<TableLds*>(&stage[0][0]);
        build_table<256>(L, p.hist_parts, p.n_parts, p.bits);
        const unsigned long long e = L.entry[tid];
        const uint32_t ml = L.max_len;
        const unsigned long long pb = L.payload_bits;
        const uint8_t ln = L.len[tid];
        __syncthreads();
        tab[tid] = e;
        if (tid == 0) {
            s_max_len = ml;
            s_payload_bits = pb;
        }
        __syncthreads();
        if (s_group == 0) p.stream[kHeaderBytes + tid] = ln;  // the code length table of the container
    } else {
        tab[tid] = p.enc_table[tid];
        if (tid == 0) {
            s_max_len = p.ctrl->max_len;
            s_payload_bits = p.ctrl->payload_bits;
        }
        __syncthreads();
    }
    const uint32_t group = s_group;
    if (group >= p.n_groups) return;  // not reachable: the grid has n_groups workgroups
    const uint32_t ch = group * kPackWaves + (uint32_t)wave;
    const bool have = ch < p.n_chunks;
    const bool long_codes = s_max_len > 32;

    // ---- the run, and pass 1 ----
    uint32_t w[16];
#pragma unroll
    for (int q = 0; q < 16; q++) w[q] = 0;
    uint32_t cnt = 0, bits = 0;
    if (have) {
        const uint64_t c0 = (uint64_t)ch * p.chunk_syms;
        const uint64_t c1 = (c0 + p.chunk_syms < p.V) ? c0 + p.chunk_syms : p.V;
        const uint64_t r0 = c0 + (uint64_t)lane * kSubSyms;
        cnt = (r0 < c1) ? (uint32_t)((c1 - r0 < kSubSyms) ? (c1 - r0) : kSubSyms) : 0u;
        if (cnt == kSubSyms && ((uintptr_t)(p.syms + r0) & 15) == 0) {
            const uint4* src = reinterpret_cast<const uint4*>(p.syms + r0);
#pragma unroll
            for (int j = 0; j < 4; j++) {
                const uint4 v = src[j];
                w[4 * j] = v.x; w[4 * j + 1] = v.y; w[4 * j + 2] = v.z; w[4 * j + 3] = v.w;
            }
        } else {
#pragma unroll
            for (int i = 0; i < kSubSyms; i++)
                if ((uint32_t)i < cnt) w[i >> 2] |= (uint32_t)p.syms[r0 + i] << (8 * (i & 3));
        }
#pragma unroll
        for (int q = 0; q < 16; q++)
#pragma unroll
            for (int b = 0; b < 4; b++)
                if ((uint32_t)(4 * q + b) < cnt) bits += (uint32_t)(tab[(w[q] >> (8 * b)) & 255u] >> 56);
        uint16_t* sub_bits = reinterpret_cast<uint16_t*>(p.stream + p.off_sub_bits);
        if ((uint32_t)lane < p.subs_per_chunk) sub_bits[(size_t)ch * p.subs_per_chunk + lane] = (uint16_t)bits;
    }
    const uint32_t start = wave_exclusive_scan(bits, lane);
    const uint32_t total_bits = __shfl(start + bits, 63, 64);
    const uint32_t n_words = (total_bits + 31) >> 5;
    if (lane == 0) wave_words[wave] = n_words;
    __syncthreads();

    // ---- the group's first payload word ----
    if (wave == 0) {
        uint32_t agg = 0;
#pragma unroll
        for (int q = 0; q < kPackWaves; q++) agg += wave_words[q];
        uint32_t excl = 0;
        if (group == 0) {
            if (lane == 0) publish64(&p.lookback[0], kFlagInclusive | agg);
        } else {
            if (lane == 0) publish64(&p.lookback[group], kFlagAggregate | agg);
            // windows of 256 predecessors, nearest first; lane l reads four of them
            uint32_t top = group;  // predecessors [0, top) are still to be accounted for
            bool failed = false;
            while (top > 0) {
                uint32_t sum = 0;
                bool found = false;  // met a running total: everything before it is included
                bool ready = false;
                for (uint32_t tries = 0; tries < kSpinLimit; tries++) {
                    sum = 0;
                    found = false;
                    bool ok = true;
#pragma unroll
                    for (int j = 0; j < 4; j++) {
                        const uint32_t back = 4u * (uint32_t)lane + (uint32_t)j + 1u;  // distance to the predecessor
                        if (back <= top && !found) {
                            const unsigned long long e = peek64(&p.lookback[top - back]);
                            if (e == 0) ok = false;
                            sum += (uint32_t)e;
                            found = (e & kFlagInclusive) != 0;
                        }
                    }
                    if (__all(ok)) {
                        ready = true;
                        break;
                    }
                    __builtin_amdgcn_s_sleep(2);
                }
                if (!ready) {
                    failed = true;
                    break;
                }
                const unsigned long long fmask = __ballot(found);
                const int first = fmask ? (__ffsll((long long)fmask) - 1) : 64;  // lanes beyond it are not needed
                const uint32_t part = (lane <= first) ? sum : 0u;
                excl += wave_sum(part);
                if (fmask) break;
                top = (top > 256u) ? top - 256u : 0u;
            }
            if (failed) {
                if (lane == 0) p.ctrl->error = 1u;
                excl = 0;
            }
            if (lane == 0) publish64(&p.lookback[group], kFlagInclusive | (unsigned long long)(excl + agg));
        }
        if (lane == 0) s_excl = excl;
    }
    __syncthreads();
    if (!have) return;  // whole wavefront leaves; no workgroup barrier follows
    uint32_t word0 = s_excl;
    for (int q = 0; q < wave; q++) word0 += wave_words[q];
    uint32_t* chunk_off = reinterpret_cast<uint32_t*>(p.stream + kHeaderBytes + kLenTableBytes);
    if (lane == 0) {
        chunk_off[ch] = word0;
        if (ch == p.n_chunks - 1) {
            const uint64_t total_words = (uint64_t)word0 + n_words;
            chunk_off[p.n_chunks] = (uint32_t)total_words;
            Header hdr = p.hdr;
            hdr.payload_words = total_words;
            hdr.payload_bits = s_payload_bits;
            if (p.ctrl->error) hdr.magic = 0u;  // a wait gave up: the stream is not valid
            *reinterpret_cast<Header*>(p.stream) = hdr;
            if (p.out_bytes) *p.out_bytes = (uint64_t)p.off_payload + 4 * total_words;
            // alignment gaps between the sections are part of the stream: keep them zero
            for (size_t o = kHeaderBytes + kLenTableBytes + 4 * ((size_t)p.n_chunks + 1); o < p.off_sub_bits; o++)
                p.stream[o] = 0;
            for (size_t o = p.off_sub_bits + 2 * (size_t)p.n_chunks * p.subs_per_chunk; o < p.off_payload; o++)
                p.stream[o] = 0;
        }
    }

    // ---- pass 2 ----
    uint32_t* img = stage[wave];
    uint32_t* out = reinterpret_cast<uint32_t*>(p.stream + p.off_payload) + word0;
    const bool all_full = __all(cnt == (uint32_t)kSubSyms || cnt == 0u) != 0;
    for (uint32_t win = 0; win < n_words; win += kStageWords) {
        const uint32_t win_words = (n_words - win < (uint32_t)kStageWords) ? n_words - win : (uint32_t)kStageWords;
        for (uint32_t i = lane; i < win_words; i += 64) img[i] = 0u;
        // LDS operations of one wavefront complete in order: the zeros land before the ORs below
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        const uint32_t first_word = start >> 5, last_word = (start + bits + 31) >> 5;  // [first, last)
        if (cnt && bits && first_word < win + win_words && last_word > win) {
            if (long_codes) pack_run<false, true>(w, cnt, start, tab, img, win, win_words);
            else if (all_full) pack_run<true, false>(w, cnt, start, tab, img, win, win_words);
            else pack_run<false, false>(w, cnt, start, tab, img, win, win_words);
        }
        // the ORs of all lanes precede the reads below: one wavefront, LDS in order
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        for (uint32_t i = lane; i < win_words; i += 64) out[win + i] = img[i];
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}

// Table (a kernel of its own only where every pack workgroup building it would cost more than the launch)
// and packing.
hipError_t launch_coder(const uint8_t* d_syms, const Geometry& g, int bits, float delta, const CoderScratch& cs,
                        int n_parts, uint64_t* d_enc_table, uint8_t* d_stream, uint64_t* d_out_bytes,
                        hipStream_t s) {
    PackParams p;
    p.syms = d_syms;
    p.V = (uint64_t)g.P * (uint64_t)g.C;
    p.n_chunks = g.n_chunks;
    p.chunk_syms = g.chunk_syms;
    p.subs_per_chunk = g.subs_per_chunk;
    p.n_groups = cs.n_groups;
    p.bits = bits;
    p.hist_parts = cs.hist_parts;
    p.n_parts = n_parts;
    p.enc_table = d_enc_table;
    p.ctrl = cs.ctrl;
    p.lookback = cs.lookback;
    p.hdr = Header{};
    p.hdr.magic = kMagic;
    p.hdr.version = 1;
    p.hdr.bits = (uint8_t)bits;
    p.hdr.C = (uint32_t)g.C;
    p.hdr.px_per_chunk = g.px_per_chunk;
    p.hdr.P = (uint64_t)g.P;
    p.hdr.n_chunks = g.n_chunks;
    p.hdr.sub_syms = kSubSyms;
    p.hdr.delta = delta;
    p.hdr.subs_per_chunk = g.subs_per_chunk;
    p.off_sub_bits = g.off_sub_bits;
    p.off_payload = g.off_payload;
    p.stream = d_stream;
    p.out_bytes = d_out_bytes;
    static const char* knob = getenv("FMTC_TABLE_IN_PACK");
    const bool build_in_pack = knob ? (knob[0] == '1') : cs.n_groups <= 512;
    if (!build_in_pack) {
        hipError_t e = launch(K_TABLE, k_huffman_table, dim3(1), dim3(1024), 0, s, (const uint32_t*)cs.hist_parts,
                              n_parts, bits, (uint32_t*)nullptr, d_enc_table, d_stream + kHeaderBytes, cs.ctrl);
        if (e != hipSuccess) return e;
        return launch(K_PACK, k_pack<false>, dim3(cs.n_groups), dim3(256), 0, s, p);
    }
    return launch(K_PACK, k_pack<true>, dim3(cs.n_groups), dim3(256), 0, s, p);
}

}  // namespace fmtc
