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
    __attribute__((aligned(16))) uint32_t h[256];
    uint32_t weight[256];       // leaf weights in (count, symbol) order
    uint32_t children[256];     // per merge: node ids of the two children (leaf i: i, internal j: 256 + j)
    uint16_t leaf_parent[256];  // merge that consumed each sorted leaf
    uint16_t int_parent[256];   // ... each internal node (numbered in creation order); then its 2^r-th ancestor
    uint16_t depth[256];        // of the internal nodes
    uint8_t len_sorted[256];    // code length of the sorted leaves
    uint32_t rank[256];         // position of every used symbol in (count, symbol) order
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

// LDS traffic of one wavefront completes in order; this keeps the compiler from moving it across the point
__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// The merge loop is serial by nature (n-1 steps).  It runs in one wavefront with the two queues held in
// registers across the lanes and all control in scalar registers, without branches: queue slots that hold
// nothing (leaves past n, nodes not made yet) weigh "infinity", which no node that can still be picked does
// (V < 2^32), and 64 * NV >= n + 2 keeps every index read inside the registers.
template <int NV>
__device__ __forceinline__ void huffman_merge(TableLds& L, int lane, int n) {
    uint32_t lw[NV], iw[NV], ch[NV];
#pragma unroll
    for (int j = 0; j < NV; j++) {
        lw[j] = (64 * j + lane < n) ? L.weight[64 * j + lane] : kInf;
        iw[j] = kInf;
        ch[j] = 0;
    }
    int nl = 0, ni = 0;
    for (int made = 0; made < n - 1; made++) {
        const uint32_t l0 = lane_get<NV>(lw, nl), l1 = lane_get<NV>(lw, nl + 1);
        const uint32_t i0 = lane_get<NV>(iw, ni), i1 = lane_get<NV>(iw, ni + 1);
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
    for (int j = 0; j < NV; j++)
        if (64 * j + lane < 256) L.children[64 * j + lane] = ch[j];
}

// The same loop for at most 64 used symbols (one register per queue), written out by hand: the compiler's
// version moves the wavefront-uniform flags through vector registers, which puts several vector-to-scalar
// round trips into every step of a loop that is one long dependency chain.  Registers only; the trip count is
// n - 1.  Lane m of the result holds the number of leaves consumed before merge m, which fixes the two
// children of every merge: merges take the queues' heads, and 2m nodes are gone before merge m.
__device__ __forceinline__ void huffman_merge_small(TableLds& L, int lane, int n) {
    const uint32_t lw = (lane < n) ? L.weight[lane] : kInf;
    uint32_t iw = kInf, rec = 0;
    const uint32_t n1 = (uint32_t)__builtin_amdgcn_readfirstlane(n - 1);
    const uint32_t nn = (uint32_t)__builtin_amdgcn_readfirstlane(n);
    uint32_t nl, ni, made, t0, t1, l0, l1, i0, i1, x, y, wa, wb, k, w, m0save;
    asm volatile(
        "s_mov_b32 %[m0save], m0\n\t"
        "s_mov_b32 %[nl], 0\n\t"
        "s_mov_b32 %[ni], 0\n\t"
        "s_mov_b32 %[made], 0\n"
        "1:\n\t"
        "s_mov_b32 m0, %[made]\n\t"
        "s_add_u32 %[t0], %[nl], 1\n\t"
        "s_add_u32 %[t1], %[ni], 1\n\t"
        "v_readlane_b32 %[l0], %[lw], %[nl]\n\t"
        "v_readlane_b32 %[i0], %[iw], %[ni]\n\t"
        "v_readlane_b32 %[l1], %[lw], %[t0]\n\t"
        "v_readlane_b32 %[i1], %[iw], %[t1]\n\t"
        "s_nop 3\n\t"
        "s_cmp_lt_u32 %[nl], %[n]\n\t"           // a queue that has run out shows "infinity"
        "s_cselect_b32 %[l0], %[l0], -1\n\t"
        "s_cmp_lt_u32 %[t0], %[n]\n\t"
        "s_cselect_b32 %[l1], %[l1], -1\n\t"
        "s_cmp_le_u32 %[l0], %[i0]\n\t"          // first pick: a leaf wins a tie
        "s_cselect_b32 %[x], %[l1], %[l0]\n\t"   // heads after the first pick
        "s_cselect_b32 %[y], %[i0], %[i1]\n\t"
        "s_cselect_b32 %[wa], %[l0], %[i0]\n\t"
        "s_cselect_b32 %[k], 1, 0\n\t"
        "s_cmp_le_u32 %[x], %[y]\n\t"            // second pick
        "s_cselect_b32 %[wb], %[x], %[y]\n\t"
        "s_addc_u32 %[k], %[k], 0\n\t"           // leaves taken by this merge
        "v_writelane_b32 %[rec], %[nl], m0\n\t"
        "s_add_u32 %[w], %[wa], %[wb]\n\t"
        "s_sub_u32 %[t0], 2, %[k]\n\t"
        "v_writelane_b32 %[iw], %[w], m0\n\t"
        "s_add_u32 %[nl], %[nl], %[k]\n\t"
        "s_add_u32 %[ni], %[ni], %[t0]\n\t"
        "s_add_u32 %[made], %[made], 1\n\t"
        "s_cmp_lt_u32 %[made], %[n1]\n\t"
        "s_cbranch_scc1 1b\n\t"
        "s_mov_b32 m0, %[m0save]\n\t"
        : [rec] "+v"(rec), [iw] "+v"(iw), [nl] "=&s"(nl), [ni] "=&s"(ni), [made] "=&s"(made), [t0] "=&s"(t0),
          [t1] "=&s"(t1), [l0] "=&s"(l0), [l1] "=&s"(l1), [i0] "=&s"(i0), [i1] "=&s"(i1), [x] "=&s"(x),
          [y] "=&s"(y), [wa] "=&s"(wa), [wb] "=&s"(wb), [k] "=&s"(k), [w] "=&s"(w), [m0save] "=&s"(m0save)
        : [lw] "v"(lw), [n1] "s"(n1), [n] "s"(nn)
        : "scc");
    // children of merge m (lane m): leaves [nlb, nla), internal nodes [2m - nlb, 2(m+1) - nla)
    const uint32_t nlb = rec;
    uint32_t nla = __shfl_down(rec, 1, 64);
    if (lane >= n - 2) nla = (uint32_t)n;  // the last merge leaves no leaf behind
    const uint32_t kk = nla - nlb, nib = 2u * (uint32_t)lane - nlb;
    const uint32_t ida = kk >= 1 ? nlb : 256u + nib;
    const uint32_t idb = kk == 2 ? nlb + 1u : (kk == 1 ? 256u + nib : 256u + nib + 1u);
    L.children[lane] = ida | (idb << 16);
}

// Sum of the partial histograms into L.h.  All THREADS threads of the workgroup call it; ends with a barrier.
template <int THREADS>
__device__ __forceinline__ void sum_partials(TableLds& L, const uint32_t* __restrict__ hist_parts, int n_parts,
                                             int bits) {
    const int tid = threadIdx.x;
    const int K = 1 << bits;
    if (tid < 256) {
        L.h[tid] = 0u;
        L.rank[tid] = 0u;
    }
    __syncthreads();
    // a thread owns four neighbouring bins of every rstep-th row; sixteen independent 16-byte loads in flight
    const int tpr = K / 4, col = tid % tpr, row0 = tid / tpr, rstep = THREADS / tpr;
    const uint4* rows = reinterpret_cast<const uint4*>(hist_parts);
    uint4 acc = make_uint4(0, 0, 0, 0);
    int q = row0;
    for (; q + 15 * rstep < n_parts; q += 16 * rstep) {
        uint4 v[16];
#pragma unroll
        for (int j = 0; j < 16; j++) v[j] = rows[(size_t)(q + j * rstep) * tpr + col];
#pragma unroll
        for (int j = 0; j < 16; j++) {
            acc.x += v[j].x; acc.y += v[j].y; acc.z += v[j].z; acc.w += v[j].w;
        }
    }
    if (q < n_parts) {  // the rest, still all in flight together
        uint4 v[15];
#pragma unroll
        for (int j = 0; j < 15; j++)
            v[j] = (q + j * rstep < n_parts) ? rows[(size_t)(q + j * rstep) * tpr + col] : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int j = 0; j < 15; j++) {
            acc.x += v[j].x; acc.y += v[j].y; acc.z += v[j].z; acc.w += v[j].w;
        }
        q = n_parts;
    }
    for (; q < n_parts; q += rstep) {
        const uint4 v = rows[(size_t)q * tpr + col];
        acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    if (acc.x) atomicAdd(&L.h[4 * col], acc.x);
    if (acc.y) atomicAdd(&L.h[4 * col + 1], acc.y);
    if (acc.z) atomicAdd(&L.h[4 * col + 2], acc.z);
    if (acc.w) atomicAdd(&L.h[4 * col + 3], acc.w);
    __syncthreads();
}

// Position of every used symbol in (count, symbol) order, into L.rank (zero on entry): the comparisons are shared
// out over all wavefronts of the workgroup, wavefront w taking the w-th slice of the symbols to compare against.
// All THREADS threads call it, after sum_partials; ends with a barrier.
template <int THREADS>
__device__ __forceinline__ void rank_symbols(TableLds& L, int bits) {
    constexpr int NW = THREADS / 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int K = 1 << bits;
    const int per = (K + NW - 1) / NW;
    const int t0 = wave * per, t1 = (t0 + per < K) ? t0 + per : K;
    for (int s = lane; s < K; s += 64) {
        const uint32_t cnt = L.h[s];
        uint32_t r = 0;
        for (int t = t0; t < t1; t++) {
            const uint32_t o = L.h[t];  // same address in all lanes: a broadcast
            r += (o != 0 && (o < cnt || (o == cnt && t < s))) ? 1u : 0u;
        }
        if (r && cnt) atomicAdd(&L.rank[s], r);
    }
    __syncthreads();
}

// What the table build leaves for its caller.
struct TableOut {
    unsigned long long* entry;  // [256] (LDS): bit-reversed code | length << 56
    uint32_t max_len;
    unsigned long long payload_bits;
};

// Canonical codes from code lengths (len[j] of symbol 64 j + lane, 0 = unused; max_len the longest, the same in
// every lane): codes of one length are numbered in symbol order, shorter codes first.  One wavefront; entry[] (256
// words, LDS or global) is written whole.
template <int NVS>
__device__ __forceinline__ void canonical_entries(const uint32_t (&len)[NVS], int lane, uint32_t max_len,
                                                  unsigned long long* entry_out) {
    uint32_t before[NVS];
#pragma unroll
    for (int j = 0; j < NVS; j++) before[j] = 0;
    // lane q ends up with the number of codes of length q
    uint32_t my_count = 0;
    for (uint32_t q = 1; q <= max_len; q++) {
        uint32_t total = 0;
#pragma unroll
        for (int j = 0; j < NVS; j++) {
            const unsigned long long m = __ballot(len[j] == q);
            if (len[j] == q) before[j] = total + (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
            total += (uint32_t)__popcll(m);
        }
        if ((uint32_t)lane == q) my_count = total;
    }
    // first canonical code of every length: code(l) = sum_{j<l} count(j) << (l-j), i.e. the running sum of
    // count(j) * 2^(48-j) shifted down to l bits
    const bool in = lane >= 1 && lane <= kMaxLen;
    const unsigned long long w = (unsigned long long)my_count << (in ? kMaxLen - lane : 0);
    const unsigned long long incl = wave_inclusive_scan64(w, lane);
    const unsigned long long first_code = in ? ((incl - w) >> (kMaxLen - lane)) : 0ull;
#pragma unroll
    for (int j = 0; j < NVS; j++) {
        const unsigned long long fc = __shfl(first_code, (int)len[j], 64);
        unsigned long long entry = 0;
        if (len[j]) {
            const unsigned long long code = fc + (unsigned long long)before[j];
            const unsigned long long rev = __brevll(code) >> (64 - len[j]);  // stream order: least significant bit first
            entry = rev | ((unsigned long long)len[j] << 56);
        }
        entry_out[64 * j + lane] = entry;
    }
    if (NVS < 4)
        for (int s = 64 * NVS + lane; s < 256; s += 64) entry_out[s] = 0ull;
}

// Code table from the histogram L.h.  Runs in ONE wavefront (64 lanes, `lane`), no workgroup barrier inside;
// lane l owns symbols l, l + 64, ... (NVS = alphabet size / 64, at least 1).  Every lane returns the same
// max_len and payload_bits; entry[] is complete when the function returns (for this wavefront).
template <int NVS>
__device__ __forceinline__ void table_from_hist(TableLds& L, int lane, int K, TableOut& out) {
    uint32_t cnt[NVS], rank[NVS];
#pragma unroll
    for (int j = 0; j < NVS; j++) {
        cnt[j] = (64 * j + lane < K) ? L.h[64 * j + lane] : 0u;
        rank[j] = (64 * j + lane < K) ? L.rank[64 * j + lane] : 0u;  // made by rank_symbols
    }
    int n = 0;
#pragma unroll
    for (int j = 0; j < NVS; j++) {
        n += __popcll(__ballot(cnt[j] != 0));
        if (cnt[j]) L.weight[rank[j]] = cnt[j];
    }
    n = __builtin_amdgcn_readfirstlane(n);
    wave_sync();
    if (n >= 2) {
        if (n <= 64) huffman_merge_small(L, lane, n);
        else if (n <= 126) huffman_merge<2>(L, lane, n);
        else if (n <= 254) huffman_merge<4>(L, lane, n);
        else huffman_merge<5>(L, lane, n);
        wave_sync();
        const int root = n - 2;
        for (int m = lane; m < n - 1; m += 64) {
            const uint32_t c = L.children[m];
            const uint32_t a = c & 0xffffu, b = c >> 16;
            if (a < 256u) L.leaf_parent[a] = (uint16_t)m; else L.int_parent[a - 256u] = (uint16_t)m;
            if (b < 256u) L.leaf_parent[b] = (uint16_t)m; else L.int_parent[b - 256u] = (uint16_t)m;
            L.depth[m] = (m == root) ? 0 : 1;
        }
        if (lane == 0) L.int_parent[root] = (uint16_t)root;
        wave_sync();
        // depth of every internal node: distance to its 2^r-th ancestor, doubled until all reach the root
        for (int r = 1; r < n - 1; r <<= 1) {
            uint32_t d[4], pp[4];
#pragma unroll
            for (int j = 0; j < 4; j++) {
                const int m = 64 * j + lane;
                if (m < n - 1) {
                    const uint32_t par = L.int_parent[m];
                    d[j] = (uint32_t)L.depth[m] + (uint32_t)L.depth[par];
                    pp[j] = L.int_parent[par];
                }
            }
            wave_sync();
#pragma unroll
            for (int j = 0; j < 4; j++) {
                const int m = 64 * j + lane;
                if (m < n - 1) {
                    L.depth[m] = (uint16_t)d[j];
                    L.int_parent[m] = (uint16_t)pp[j];
                }
            }
            wave_sync();
        }
        for (int i = lane; i < n; i += 64) {
            uint32_t l = (uint32_t)L.depth[L.leaf_parent[i]] + 1u;
            // more than kMaxLen is unreachable for V < 2^32 (depth d needs a total count >= Fibonacci(d+2))
            L.len_sorted[i] = (uint8_t)(l > (uint32_t)kMaxLen ? (uint32_t)kMaxLen : l);
        }
    } else if (lane == 0) {
        L.len_sorted[0] = 1;  // a single used symbol gets the one-bit code 0
    }
    wave_sync();
    uint32_t len[NVS];
    uint32_t max_len = 0;
    unsigned long long pbits = 0;
#pragma unroll
    for (int j = 0; j < NVS; j++) {
        len[j] = cnt[j] ? (uint32_t)L.len_sorted[rank[j]] : 0u;
        max_len = len[j] > max_len ? len[j] : max_len;
        pbits += (unsigned long long)cnt[j] * len[j];
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const uint32_t t = __shfl_xor(max_len, o, 64);
        max_len = t > max_len ? t : max_len;
        pbits += __shfl_xor(pbits, o, 64);
    }
    max_len = (uint32_t)__builtin_amdgcn_readfirstlane((int)max_len);
    canonical_entries<NVS>(len, lane, max_len, out.entry);
    out.max_len = max_len;
    out.payload_bits = pbits;
    wave_sync();
}

__device__ __forceinline__ void table_from_hist_any(TableLds& L, int lane, int bits, TableOut& out) {
    if (bits <= 6) table_from_hist<1>(L, lane, 1 << bits, out);
    else if (bits == 7) table_from_hist<2>(L, lane, 128, out);
    else table_from_hist<4>(L, lane, 256, out);
}

__global__ __launch_bounds__(1024) void k_huffman_table(const uint32_t* __restrict__ hist_parts, int n_parts,
                                                        int bits, uint32_t* __restrict__ hist_out,
                                                        uint64_t* __restrict__ enc_table,
                                                        uint8_t* __restrict__ len_table,
                                                        CoderCtrl* __restrict__ ctrl, uint32_t add_each) {
    __shared__ TableLds L;
    __shared__ unsigned long long entry[256];
    sum_partials<1024>(L, hist_parts, n_parts, bits);
    if (add_each) {  // a table for tensors to come: every symbol of the alphabet gets a code
        if ((int)threadIdx.x < (1 << bits)) L.h[threadIdx.x] += add_each;
        __syncthreads();
    }
    rank_symbols<1024>(L, bits);
    const int tid = threadIdx.x;
    if (tid < 64) {
        TableOut out;
        out.entry = entry;
        table_from_hist_any(L, tid, bits, out);
        if (tid == 0 && ctrl) {
            ctrl->max_len = out.max_len;
            ctrl->payload_bits = out.payload_bits;
        }
    }
    __syncthreads();
    if (tid < 256) {
        if (hist_out) hist_out[tid] = L.h[tid];
        if (enc_table) enc_table[tid] = entry[tid];
        if (len_table) len_table[tid] = (uint8_t)(entry[tid] >> 56);
    }
}

// Code table of given lengths (a complete prefix code over the 2^bits symbols; the host has checked that).
__global__ __launch_bounds__(64) void k_table_from_lengths(const uint8_t* __restrict__ len_table, int bits,
                                                           uint64_t* __restrict__ enc_table) {
    const int lane = threadIdx.x, K = 1 << bits;
    uint32_t len[4], max_len = 0;
#pragma unroll
    for (int j = 0; j < 4; j++) {
        len[j] = (64 * j + lane < K) ? (uint32_t)len_table[64 * j + lane] : 0u;
        max_len = len[j] > max_len ? len[j] : max_len;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const uint32_t t = __shfl_xor(max_len, o, 64);
        max_len = t > max_len ? t : max_len;
    }
    max_len = (uint32_t)__builtin_amdgcn_readfirstlane((int)max_len);
    canonical_entries<4>(len, lane, max_len, reinterpret_cast<unsigned long long*>(enc_table));
}

hipError_t launch_table_from_lengths(const uint8_t* d_len_table, int bits, uint64_t* d_enc_table, hipStream_t s) {
    return launch(K_TABLE, k_table_from_lengths, dim3(1), dim3(64), 0, s, d_len_table, bits, d_enc_table);
}

// Table of the summed partial histograms with `add_each` added to every symbol's count.
hipError_t launch_table_from_hist(const uint32_t* d_hist_parts, int n_parts, int bits, uint32_t add_each,
                                  uint64_t* d_enc_table, uint8_t* d_len_table, hipStream_t s) {
    return launch(K_TABLE, k_huffman_table, dim3(1), dim3(1024), 0, s, d_hist_parts, n_parts, bits,
                  (uint32_t*)nullptr, d_enc_table, d_len_table, (CoderCtrl*)nullptr, add_each);
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
// Packing.  One wavefront per chunk, in ONE pass over the symbols: the wavefront walks the
// chunk in steps of 256 consecutive symbols (lane l holds symbols 4l .. 4l+3 of the step, one
// 4-byte load), looks the codes up, joins the codes of a lane into one value of at most 64
// bits, and a prefix sum over the lanes (row shifts and row broadcasts, no LDS) gives every
// lane its bit position; the value is ORed into an LDS image of the chunk.  The prefix sum
// also yields the bit count of every run of 64 symbols, which the container stores so that 64
// lanes can decode a chunk.  (A table with codes longer than 32 bits takes one symbol per lane
// and step instead.)
// Workgroups are persistent: the grid never exceeds what the device holds at once and
// workgroup w takes the chunk groups w, w + grid, ... in turn, so every predecessor of a group
// is either finished or being worked on by a resident workgroup.  The chunk's first payload
// word is the number of words of all chunks before it: a workgroup publishes its group's word
// count and reads back over its predecessors' published counts until it meets one that is
// already a running total.  The image of the first window is built before that position is
// known and leaves with full-width stores.  A chunk larger than the image is produced in
// several windows.
// ---------------------------------------------------------------------------
constexpr int kStageWords = 2048;  // per wavefront: 64 Kbit, i.e. 16 bits/symbol over a 4096-symbol chunk
// A look-back entry: payload words in bits 0..31, bits left unused in the last words of the chunks ("slack",
// below 32 per chunk) in bits 32..61, and in bits 62..63 whether it covers one group or everything up to it.
constexpr unsigned long long kFlagAggregate = 1ull << 62, kFlagInclusive = 2ull << 62;
constexpr uint32_t kSlackMask = 0x3fffffffu;
enum PackMode { kPackBuild = 0, kPackTable = 1, kPackStatic = 2 };  // who made the table: this kernel from the
                                                                     // histogram, k_huffman_table, or the caller
constexpr int kLook = 4;  // look-back entries a lane reads per poll (each is an uncached device-scope load: wider windows cost more than the extra round trips they save)
constexpr uint32_t kSpinLimit = 1u << 22;  // polls before a wait gives up (seconds; never reached unless the
                                           // workspace is overwritten while the kernel runs)

struct PackParams {
    const uint8_t* syms;
    uint64_t V;
    uint32_t n_chunks, chunk_syms, subs_per_chunk, n_groups;
    int bits;
    const uint32_t* hist_parts;  // kPackBuild: partial histograms to build the table from
    int n_parts;
    const uint64_t* enc_table;   // otherwise: the table (k_huffman_table's, or a static one)
    uint32_t static_max_len;     // kPackStatic: longest code of the table
    CoderCtrl* ctrl;
    unsigned long long* lookback;
    Header hdr;
    size_t off_sub_bits, off_payload;
    uint64_t cap_words;          // payload words the output buffer has room for
    uint8_t* stream;
    uint64_t* out_bytes;
};

// x + (x of the lane the control word names), 0 where that lane does not exist or the row is masked out
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_add(uint32_t x) {
    return x + (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, ROW_MASK, 0xf, false);
}
// Inclusive prefix sum over the 64 lanes.  row: the sum within the lane's row of 16 lanes (lane 15 of a row
// holds the row total); half: the sum within the lane's half of the wavefront (lanes 31 and 63 hold the totals).
__device__ __forceinline__ uint32_t wave_inclusive_scan_rows(uint32_t v, uint32_t& row, uint32_t& half) {
    v = dpp_add<0x111, 0xf>(v);  // row_shr:1
    v = dpp_add<0x112, 0xf>(v);  // row_shr:2
    v = dpp_add<0x114, 0xf>(v);  // row_shr:4
    v = dpp_add<0x118, 0xf>(v);  // row_shr:8
    row = v;
    v = dpp_add<0x142, 0xa>(v);  // row_bcast:15 into rows 1 and 3
    half = v;
    v = dpp_add<0x143, 0xc>(v);  // row_bcast:31 into rows 2 and 3
    return v;
}

// ORs the bits of `c` (zero above its length) into the image at bit `pos` of the chunk.  The image is followed
// by spare words: ORing zeros does no harm, so nothing here branches per lane.
//   FIRST window: positions are cut off at the end of the image, what lies beyond lands in the spare words;
//   later windows (rare): every word is checked against the window.
// third: some lane's bits reach into a third word (wavefront-uniform).
template <bool FIRST>
__device__ __forceinline__ void place_bits(unsigned long long c, uint32_t pos, uint32_t* img, uint32_t win,
                                           uint32_t win_words, bool third) {
    const unsigned long long t0 = (unsigned long long)(uint32_t)c << (pos & 31u);
    const unsigned long long t1 = ((unsigned long long)(uint32_t)(c >> 32) << (pos & 31u)) | (t0 >> 32);
    if constexpr (FIRST) {
        const uint32_t widx = (pos < (uint32_t)kStageWords * 32u ? pos : (uint32_t)kStageWords * 32u) >> 5;
        atomicOr(&img[widx], (uint32_t)t0);
        atomicOr(&img[widx + 1u], (uint32_t)t1);
        if (third) atomicOr(&img[widx + 2u], (uint32_t)(t1 >> 32));
    } else {
        const uint32_t rel = (pos >> 5) - win;
        const uint32_t i0 = rel < win_words ? rel : (uint32_t)kStageWords;
        const uint32_t i1 = rel + 1u < win_words ? rel + 1u : (uint32_t)kStageWords;
        const uint32_t i2 = rel + 2u < win_words ? rel + 2u : (uint32_t)kStageWords;
        atomicOr(&img[i0], (uint32_t)t0);
        atomicOr(&img[i1], (uint32_t)t1);
        atomicOr(&img[i2], (uint32_t)(t1 >> 32));
    }
}

// One chunk (`clen` symbols, in w: register q of lane l holds symbols 256q + 4l .. + 3) into the window
// [win, win + win_words) of its image.  Returns the chunk's code bits; with run_bits != NULL also stores the bit
// count of each of the n_runs runs of 64 symbols there.
//   LONG = false (codes of at most 32 bits): a lane joins its four symbols of a step; in the rare step where
//   some lane's four codes exceed 64 bits the wavefront places them as two halves.
//   LONG = true: one symbol per lane and step.
// The loop over the registers is a real loop (the register file has no indexed access: the working copy is
// rotated by four registers per turn instead).
template <bool LONG, bool FIRST>
__device__ __forceinline__ uint32_t pack_chunk(const uint32_t (&w)[16], uint32_t clen,
                                               const unsigned long long* tab, uint32_t* img, uint32_t win,
                                               uint32_t win_words, int lane, uint16_t* run_bits, uint32_t n_runs) {
    uint32_t r[16];
#pragma unroll
    for (int q = 0; q < 16; q++) r[q] = w[q];
    uint32_t base = 0;  // code bits of the symbols before this step
    const uint32_t n_regs = (clen + 255u) >> 8;
#pragma unroll 1
    for (uint32_t q4 = 0; q4 < n_regs; q4 += 4) {
#pragma unroll
        for (int k = 0; k < 4; k++) {
            const uint32_t q = q4 + k;
            if (q >= n_regs) break;  // wavefront-uniform
            if constexpr (!LONG) {
                const uint32_t first = 256u * q + 4u * (uint32_t)lane;  // this lane's first symbol
                unsigned long long e[4];
                if (256u * (q + 1) <= clen) {
#pragma unroll
                    for (int i = 0; i < 4; i++) e[i] = tab[(r[k] >> (8 * i)) & 255u];
                } else {
#pragma unroll
                    for (int i = 0; i < 4; i++) e[i] = (first + i < clen) ? tab[(r[k] >> (8 * i)) & 255u] : 0ull;
                }
                const uint32_t l0 = (uint32_t)(e[0] >> 56), l1 = (uint32_t)(e[1] >> 56);
                const uint32_t l2 = (uint32_t)(e[2] >> 56), l3 = (uint32_t)(e[3] >> 56);
                const unsigned long long lo = (unsigned long long)(uint32_t)e[0] | ((unsigned long long)(uint32_t)e[1] << l0);
                const unsigned long long hi = (unsigned long long)(uint32_t)e[2] | ((unsigned long long)(uint32_t)e[3] << l2);
                const uint32_t l01 = l0 + l1, len = l01 + l2 + l3;
                uint32_t row, half;
                const uint32_t incl = wave_inclusive_scan_rows(len, row, half);
                const uint32_t pos = base + incl - len;
                if (__builtin_expect(__any(len > 64u), 0)) {
                    place_bits<FIRST>(lo, pos, img, win, win_words, true);
                    place_bits<FIRST>(hi, pos + l01, img, win, win_words, true);
                } else {
                    // l01 = 64 leaves no bits in hi
                    const unsigned long long c = lo | (hi << (l01 & 63u));
                    place_bits<FIRST>(c, pos, img, win, win_words, __any(len + (pos & 31u) > 64u) != 0);
                }
                if (run_bits) {  // a run of 64 symbols is a row of 16 lanes
                    const uint32_t run = 4u * q + (uint32_t)(lane >> 4);
                    if ((lane & 15) == 15 && run < n_runs) run_bits[run] = (uint16_t)row;
                }
                base += (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
            } else {
#pragma unroll
                for (int u = 0; u < 4; u++) {
                    // symbol 64u + l of the step sits in lane 16u + l/4, byte l%4
                    const uint32_t first = 256u * q + 64u * u + (uint32_t)lane;
                    const uint32_t v = (uint32_t)__shfl((int)r[k], 16 * u + (lane >> 2), 64) >> (8 * (lane & 3));
                    const unsigned long long e0 = (first < clen) ? tab[v & 255u] : 0ull;
                    const uint32_t len = (uint32_t)(e0 >> 56);
                    uint32_t row, half;
                    const uint32_t incl = wave_inclusive_scan_rows(len, row, half);
                    place_bits<FIRST>(e0 & 0x00ffffffffffffffull, base + incl - len, img, win, win_words, true);
                    const uint32_t run = 4u * q + (uint32_t)u;
                    if (run_bits && lane == 63 && run < n_runs) run_bits[run] = (uint16_t)incl;
                    base += (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
                }
            }
        }
#pragma unroll
        for (int k = 0; k < 12; k++) r[k] = r[k + 4];
    }
    // runs of a short chunk that hold no symbol (the steps above stop at the chunk's end)
    if (run_bits)
        for (uint32_t run = 4u * n_regs + (uint32_t)lane; run < n_runs; run += 64) run_bits[run] = 0;
    return base;
}

// kPackWaves chunks per group: one wavefront per chunk.
template <int MODE>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 4))) void k_pack(PackParams p) {
    static_assert(kPackWaves == 4, "one chunk per wavefront of the 256-thread workgroup");
    __shared__ unsigned long long tab[256];
    __shared__ __align__(16) uint32_t stage[kPackWaves][kStageWords + 4];  // image + the spare word
    __shared__ uint32_t wave_words[kPackWaves], wave_slack[kPackWaves];
    __shared__ uint32_t s_excl, s_excl_slack, s_max_len;
    __shared__ unsigned long long s_payload_bits;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wavefront-uniform by construction
    const bool aligned4 = (p.chunk_syms & 3u) == 0;  // every chunk starts on a 4-byte boundary of the symbols

    // the symbols of a chunk: register q of lane l holds symbols 256q + 4l .. + 3 (zero past the chunk's end)
    auto chunk_len = [&](uint32_t ch) -> uint32_t {
        if (ch >= p.n_chunks) return 0u;
        const uint64_t c0 = (uint64_t)ch * p.chunk_syms;
        return (uint32_t)((p.V - c0 < p.chunk_syms) ? (p.V - c0) : p.chunk_syms);
    };
    auto load_chunk = [&](uint32_t ch, uint32_t (&w)[16]) {
        const uint32_t clen = chunk_len(ch);
        const uint8_t* src = p.syms + (uint64_t)ch * p.chunk_syms;
        if (aligned4) {
#pragma unroll
            for (int q = 0; q < 16; q++) {
                const uint32_t o = 256u * q + 4u * (uint32_t)lane;
                w[q] = (o + 4u <= clen) ? *reinterpret_cast<const uint32_t*>(src + o) : 0u;
            }
            if (clen & 3u) {  // the last, partial word of the tensor
                const uint32_t t = clen & ~3u;
                uint32_t v = 0;
                if ((uint32_t)lane == ((t >> 2) & 63u))
                    for (uint32_t i = 0; i < (clen & 3u); i++) v |= (uint32_t)src[t + i] << (8 * i);
#pragma unroll
                for (int q = 0; q < 16; q++)
                    if ((uint32_t)q == (t >> 8)) w[q] |= v;
            }
        } else {
#pragma unroll
            for (int q = 0; q < 16; q++) {
                const uint32_t o = 256u * q + 4u * (uint32_t)lane;
                w[q] = 0u;
#pragma unroll
                for (int i = 0; i < 4; i++)
                    if (o + i < clen) w[q] |= (uint32_t)src[o + i] << (8 * i);
                __builtin_amdgcn_sched_barrier(0);  // one register's loads at a time: this path is rare
            }
        }
    };
    uint32_t w[16];
    uint32_t group = blockIdx.x;  // the grid never has more workgroups than groups
    load_chunk(group * kPackWaves + (uint32_t)wave, w);  // in flight while the table is made

    TableLds& L = *reinterpret_cast<TableLds*>(&stage[0][0]);  // shares LDS with the chunk images, not in use yet
    static_assert(sizeof(TableLds) <= sizeof(stage), "table scratch must fit the chunk images");
    if constexpr (MODE == kPackBuild) {
        sum_partials<256>(L, p.hist_parts, p.n_parts, p.bits);
        rank_symbols<256>(L, p.bits);
        if (wave == 0) {
            TableOut out;
            out.entry = tab;
            table_from_hist_any(L, lane, p.bits, out);
            if (lane == 0) {
                s_max_len = out.max_len;
                s_payload_bits = out.payload_bits;
            }
        }
        __syncthreads();
        if (blockIdx.x == 0) p.stream[kHeaderBytes + tid] = (uint8_t)(tab[tid] >> 56);  // the container's length table
    } else {
        tab[tid] = p.enc_table[tid];
        if (tid == 0) {
            // a static table does not know this tensor's bit count: it comes out of the look-back (see below)
            s_max_len = MODE == kPackStatic ? p.static_max_len : p.ctrl->max_len;
            s_payload_bits = MODE == kPackStatic ? 0ull : p.ctrl->payload_bits;
        }
        __syncthreads();
        if (MODE == kPackStatic && blockIdx.x == 0) p.stream[kHeaderBytes + tid] = (uint8_t)(tab[tid] >> 56);
    }
    const uint32_t max_len = s_max_len;
    uint32_t* img = stage[wave];
    // nobody reads the table scratch any more: the images start out clear
    for (int i = lane; i < kStageWords / 4; i += 64) reinterpret_cast<uint4*>(img)[i] = make_uint4(0u, 0u, 0u, 0u);
    wave_sync();
    uint16_t* sub_bits = reinterpret_cast<uint16_t*>(p.stream + p.off_sub_bits);
    uint32_t* chunk_off = reinterpret_cast<uint32_t*>(p.stream + kHeaderBytes + kLenTableBytes);

    for (; group < p.n_groups; group += gridDim.x) {
        const uint32_t ch = group * kPackWaves + (uint32_t)wave;
        const bool have = ch < p.n_chunks;
        const uint32_t clen = chunk_len(ch);

        // ---- the first window of the chunk's image: needs no global position ----
        // (the image is all zero here: cleared once at the start and again by whoever reads a word out)
        auto build_window = [&](uint32_t win, uint32_t win_words, uint16_t* run_bits) -> uint32_t {
            uint32_t total;
            const uint32_t n_runs = p.subs_per_chunk;
            if (win == 0) {
                if (max_len <= 32) total = pack_chunk<false, true>(w, clen, tab, img, win, win_words, lane, run_bits, n_runs);
                else total = pack_chunk<true, true>(w, clen, tab, img, win, win_words, lane, run_bits, n_runs);
            } else {
                if (max_len <= 32) total = pack_chunk<false, false>(w, clen, tab, img, win, win_words, lane, run_bits, n_runs);
                else total = pack_chunk<true, false>(w, clen, tab, img, win, win_words, lane, run_bits, n_runs);
            }
            wave_sync();  // the ORs of all lanes precede the reads that follow
            return total;
        };
        uint32_t n_words = 0, slack = 0;
        if (have) {
            const uint32_t total_bits = build_window(0, kStageWords, sub_bits + (size_t)ch * p.subs_per_chunk);
            n_words = (total_bits + 31) >> 5;
            slack = 32u * n_words - total_bits;
        }
        if (lane == 0) {
            wave_words[wave] = n_words;
            wave_slack[wave] = slack;
        }
        __syncthreads();
        uint32_t agg = 0, agg_slack = 0;
#pragma unroll
        for (int q = 0; q < kPackWaves; q++) {
            agg += wave_words[q];
            agg_slack += wave_slack[q];
        }
        if (tid == 0)
            publish64(&p.lookback[group], (group == 0 ? kFlagInclusive : kFlagAggregate) |
                                              ((unsigned long long)agg_slack << 32) | agg);

        // the next group's symbols are on their way during the wait for the position and the stores
        uint32_t wn[16];
        const uint32_t next_group = group + gridDim.x;
        if (next_group < p.n_groups) load_chunk(next_group * kPackWaves + (uint32_t)wave, wn);

        // ---- the group's first payload word: the words of all groups before it ----
        if (wave == 0 && group != 0) {
            // windows of 64 * kLook predecessors, nearest first; lane l reads kLook of them, all loads in flight
            // together
            uint32_t excl = 0, excl_slack = 0;
            uint32_t top = group;  // predecessors [0, top) are still to be accounted for
            bool failed = false;
            while (top > 0) {
                uint32_t sum = 0, ssum = 0;
                bool found = false;  // met a running total: everything before it is included
                bool ready = false;
                for (uint32_t tries = 0; tries < kSpinLimit; tries++) {
                    unsigned long long e[kLook];
#pragma unroll
                    for (int j = 0; j < kLook; j++) {
                        const uint32_t back = (uint32_t)kLook * (uint32_t)lane + (uint32_t)j + 1u;  // distance to the predecessor
                        e[j] = (back <= top) ? peek64(&p.lookback[top - back]) : kFlagAggregate;
                    }
                    sum = 0;
                    ssum = 0;
                    found = false;
                    bool ok = true;
#pragma unroll
                    for (int j = 0; j < kLook; j++) {
                        if (!found) {
                            if (e[j] == 0) ok = false;
                            sum += (uint32_t)e[j];
                            ssum += (uint32_t)(e[j] >> 32) & kSlackMask;
                            found = (e[j] & kFlagInclusive) != 0;
                        }
                    }
                    // entries behind a running total need not be there yet
                    const unsigned long long fm = __ballot(found);
                    const unsigned long long need = fm ? ((2ull << (__ffsll((long long)fm) - 1)) - 1ull) : ~0ull;
                    if ((__ballot(!ok) & need) == 0) {
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
                excl += wave_sum((lane <= first) ? sum : 0u);
                excl_slack += wave_sum((lane <= first) ? ssum : 0u);
                if (fmask) break;
                top = (top > 64u * kLook) ? top - 64u * kLook : 0u;
            }
            if (failed) {
                if (lane == 0) p.ctrl->error = 1u;
                excl = 0;
                excl_slack = 0;
            }
            if (lane == 0) {
                publish64(&p.lookback[group], kFlagInclusive | ((unsigned long long)(excl_slack + agg_slack) << 32) |
                                                  (unsigned long long)(excl + agg));
                s_excl = excl;
                s_excl_slack = excl_slack;
            }
        } else if (tid == 0) {
            s_excl = 0;
            s_excl_slack = 0;
        }
        __syncthreads();
        if (have) {
            uint32_t word0 = s_excl;
            for (int q = 0; q < wave; q++) word0 += wave_words[q];
            if (lane == 0) {
                chunk_off[ch] = word0;
                if (ch == p.n_chunks - 1) {
                    const uint64_t total_words = (uint64_t)word0 + n_words;
                    chunk_off[p.n_chunks] = (uint32_t)total_words;
                    Header hdr = p.hdr;
                    hdr.payload_words = total_words;
                    hdr.payload_bits = s_payload_bits;
                    if constexpr (MODE == kPackStatic) {
                        // every code bit of the tensor: the words of all chunks less what their last words leave unused
                        uint32_t total_slack = s_excl_slack + slack;
                        for (int q = 0; q < wave; q++) total_slack += wave_slack[q];
                        hdr.payload_bits = 32ull * total_words - total_slack;
                    }
                    // a wait gave up, or the payload outgrew the buffer (then some chunk was not written): not valid
                    if (p.ctrl->error || total_words > p.cap_words) hdr.magic = 0u;
                    *reinterpret_cast<Header*>(p.stream) = hdr;
                    if (p.out_bytes) *p.out_bytes = (uint64_t)p.off_payload + 4 * total_words;
                    // alignment gaps between the sections are part of the stream: keep them zero
                    for (size_t o = kHeaderBytes + kLenTableBytes + 4 * ((size_t)p.n_chunks + 1); o < p.off_sub_bits; o++)
                        p.stream[o] = 0;
                    for (size_t o = p.off_sub_bits + 2 * (size_t)p.n_chunks * p.subs_per_chunk; o < p.off_payload; o++)
                        p.stream[o] = 0;
                }
            }
            // ---- the image leaves with full-width stores; further windows (rare) are built and stored in turn ----
            // (An optimal code of the tensor's own histogram always fits the capacity the host checked.  Should the
            // histogram and the symbols ever disagree, nothing is written past the buffer: the stream is marked
            // invalid instead.)
            const bool fits = (uint64_t)word0 + n_words <= p.cap_words;
            if (!fits && lane == 0) p.ctrl->error = 1u;
            uint32_t* out = reinterpret_cast<uint32_t*>(p.stream + p.off_payload) + word0;
            for (uint32_t win = 0; win < n_words; win += kStageWords) {
                const uint32_t win_words = (n_words - win < (uint32_t)kStageWords) ? n_words - win : (uint32_t)kStageWords;
                if (win) build_window(win, win_words, nullptr);
                for (uint32_t i = lane; i < win_words; i += 64) {
                    if (fits) out[win + i] = img[i];
                    img[i] = 0u;
                }
                wave_sync();  // the image is read and clear before the next window or chunk writes it
            }
        }
        __syncthreads();  // wave_words, wave_slack and s_excl* are rewritten by the next group
#pragma unroll
        for (int q = 0; q < 16; q++) w[q] = wn[q];
    }
}

// Number of workgroups of the pack kernel the device holds at once (queried once per kernel variant).
template <int MODE>
static int pack_resident_groups() {
    static int cached = 0;
    if (cached) return cached;
    int dev = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_pack<MODE>, 256, 0) != hipSuccess || cus < 1 ||
        per_cu < 1)
        return 64;  // conservative: any device this library runs on holds 64 workgroups
    if (per_cu > 4) per_cu = 4;
    cached = cus * per_cu;
    return cached;
}

// Table (a kernel of its own only where every pack workgroup building it would cost more than the launch)
// and packing.
static PackParams pack_params(const uint8_t* d_syms, const Geometry& g, int bits, float delta, const CoderScratch& cs,
                              int n_parts, const uint64_t* d_enc_table, uint8_t* d_stream, uint64_t cap_words,
                              uint64_t* d_out_bytes) {
    PackParams p;
    p.cap_words = cap_words;
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
    p.static_max_len = 0;
    return p;
}

hipError_t launch_coder(const uint8_t* d_syms, const Geometry& g, int bits, float delta, const CoderScratch& cs,
                        int n_parts, uint64_t* d_enc_table, uint8_t* d_stream, uint64_t cap_words,
                        uint64_t* d_out_bytes, hipStream_t s) {
    PackParams p = pack_params(d_syms, g, bits, delta, cs, n_parts, d_enc_table, d_stream, cap_words, d_out_bytes);
    static const char* knob = getenv("FMTC_TABLE_IN_PACK");
    // every pack workgroup sums the partial histograms itself while that is at most 64 KB to read
    const bool build_in_pack = knob ? (knob[0] == '1') : ((size_t)n_parts << bits) * 4 <= 64 * 1024;
    if (!build_in_pack) {
        hipError_t e = launch(K_TABLE, k_huffman_table, dim3(1), dim3(1024), 0, s, (const uint32_t*)cs.hist_parts,
                              n_parts, bits, (uint32_t*)nullptr, d_enc_table, d_stream + kHeaderBytes, cs.ctrl, 0u);
        if (e != hipSuccess) return e;
        const uint32_t cap = (uint32_t)pack_resident_groups<kPackTable>();
        return launch(K_PACK, k_pack<kPackTable>, dim3(cs.n_groups < cap ? cs.n_groups : cap), dim3(256), 0, s, p);
    }
    const uint32_t cap = (uint32_t)pack_resident_groups<kPackBuild>();
    return launch(K_PACK, k_pack<kPackBuild>, dim3(cs.n_groups < cap ? cs.n_groups : cap), dim3(256), 0, s, p);
}

// Packing with a table fixed beforehand (one code for every symbol of the alphabet): no histogram, no table build.
// The coder's counters must be clear (the kernel that made the symbols clears them).
hipError_t launch_coder_static(const uint8_t* d_syms, const Geometry& g, int bits, float delta, const CoderScratch& cs,
                               const uint64_t* d_enc_table, uint32_t max_len, uint8_t* d_stream, uint64_t cap_words,
                               uint64_t* d_out_bytes, hipStream_t s) {
    PackParams p = pack_params(d_syms, g, bits, delta, cs, 0, d_enc_table, d_stream, cap_words, d_out_bytes);
    p.static_max_len = max_len;
    const uint32_t cap = (uint32_t)pack_resident_groups<kPackStatic>();
    return launch(K_PACK, k_pack<kPackStatic>, dim3(cs.n_groups < cap ? cs.n_groups : cap), dim3(256), 0, s, p);
}

}  // namespace fmtc
