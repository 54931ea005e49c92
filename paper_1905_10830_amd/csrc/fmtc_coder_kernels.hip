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
#include <atomic>

#include "fmtc_device.h"
#include "fmtc_internal.h"
#include "fmtc_pack_device.h"

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
    uint32_t weight[260];       // leaf weights in (count, symbol) order (4 spare entries: reads just past the end)
    uint32_t children[256];     // per merge: node ids of the two children (leaf i: i, internal j: 256 + j)
    uint16_t leaf_parent[256];  // merge that consumed each sorted leaf
    uint16_t int_parent[256];   // ... each internal node (numbered in creation order); then its 2^r-th ancestor
    uint16_t depth[256];        // of the internal nodes
    uint8_t len_sorted[256];    // code length of the sorted leaves
    uint32_t rank[260];         // position of every used symbol in (count, symbol) order; reused by the serial merge
};

// LDS traffic of one wavefront completes in order; this keeps the compiler from moving it across the point
__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// The merge loop is serial by nature (n - 1 steps).
// More than 64 used symbols: the queues in LDS and the whole loop in ONE lane.  A step is four LDS reads in flight
// together, a dozen dependent operations and two LDS writes; spreading the queues over the lanes' registers
// instead costs four cross-lane reads per queue entry and, measured, several times as long per step.
// Internal node weights go where the ranks were (the caller holds those in registers by now).
__device__ __forceinline__ void huffman_merge_serial(TableLds& L, int lane, int n) {
    uint32_t* iw = L.rank;
    for (int i = lane; i < 260; i += 64) {
        iw[i] = kInf;
        if (i >= n) L.weight[i] = kInf;
    }
    wave_sync();
    if (lane == 0) {
        int nl = 0, ni = 0;
        for (int made = 0; made < n - 1; made++) {
            // a queue that has run out shows "infinity" (the arrays have spare entries behind index 255)
            const uint32_t l0 = L.weight[nl], l1 = L.weight[nl + 1];
            const uint32_t i0 = iw[ni], i1 = iw[ni + 1];
            const bool a_leaf = l0 <= i0;  // first pick: a leaf wins over an internal node of equal weight
            const uint32_t wa = a_leaf ? l0 : i0;
            const uint32_t ida = a_leaf ? (uint32_t)nl : 256u + (uint32_t)ni;
            const uint32_t ln = a_leaf ? l1 : l0, in = a_leaf ? i0 : i1;
            const int nl1 = nl + (a_leaf ? 1 : 0), ni1 = ni + (a_leaf ? 0 : 1);
            const bool b_leaf = ln <= in;
            const uint32_t wb = b_leaf ? ln : in;
            const uint32_t idb = b_leaf ? (uint32_t)nl1 : 256u + (uint32_t)ni1;
            nl = nl1 + (b_leaf ? 1 : 0);
            ni = ni1 + (b_leaf ? 0 : 1);
            iw[made] = wa + wb;
            L.children[made] = ida | (idb << 16);
        }
    }
    wave_sync();
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
#pragma unroll 16  // the reads of many steps in flight together: a step is one LDS round trip otherwise
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
// scratch64: 64 words of LDS the wavefront may use (or NULL).
template <int NVS>
__device__ __forceinline__ void canonical_entries(const uint32_t (&len)[NVS], int lane, uint32_t max_len,
                                                  unsigned long long* entry_out, uint32_t* scratch64 = nullptr) {
    uint32_t before[NVS];
#pragma unroll
    for (int j = 0; j < NVS; j++) before[j] = 0;
    // lane q ends up with the number of codes of length q
    uint32_t my_count = 0;
    if (NVS == 1 && scratch64) {
        // One symbol per lane: the lanes of equal length found with six ballots (one per bit of the length) instead
        // of a loop over the lengths; the first lane of every length hands the group's size to the lane whose
        // index is that length.
        unsigned long long same = ~0ull;
#pragma unroll
        for (int bit = 0; bit < 6; bit++) {
            const unsigned long long m = __ballot((len[0] >> bit) & 1u);
            same &= ((len[0] >> bit) & 1u) ? m : ~m;
        }
        before[0] = (uint32_t)__popcll(same & ((1ull << lane) - 1ull));
        const uint32_t group = (uint32_t)__popcll(same);
        // (lengths are at most kMaxLen < 64: the lane that holds a length's count exists)
        scratch64[lane] = 0u;
        wave_sync();
        if (len[0] && before[0] == 0) scratch64[len[0]] = group;
        wave_sync();
        const uint32_t cnt_here = scratch64[lane];
        my_count = cnt_here;
    } else {
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
        else huffman_merge_serial(L, lane, n);
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
    canonical_entries<NVS>(len, lane, max_len, out.entry, L.rank);  // (the ranks are in registers by now)
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
// Packing kernel: the table (made here, by k_huffman_table, or given), then the chunk groups
// in turn (see fmtc_pack_device.h).
// ---------------------------------------------------------------------------
// kPackWaves chunks per group: one wavefront per chunk.
template <int MODE>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 4))) void k_pack(PackParams p) {
    static_assert(kPackWaves == 4, "one chunk per wavefront of the 256-thread workgroup");
    __shared__ PackShared S;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wavefront-uniform by construction
    const bool aligned4 = (p.chunk_syms & 3u) == 0;  // every chunk starts on a 4-byte boundary of the symbols

    // Which groups a workgroup packs.  A group's position in the payload comes from the groups before it, so
    // whoever waits for one must know that its owner gets to run.  This kernel is only launched with no more
    // groups than the device holds workgroups of it, and workgroup g takes group g: within a part of the chip
    // workgroups start in index order, so the lowest unfinished group is either running or next in line for a
    // place that only other kernels' workgroups (which finish) or this kernel's finished ones can hold.  Larger
    // tensors take the kernels below (k_chunk_bits, k_chunk_scan, k_pack_at), which never wait for each other.
    uint32_t w[16];
    const uint32_t group = blockIdx.x;  // the grid never has more workgroups than groups
    load_chunk_symbols(p, group * kPackWaves + (uint32_t)wave, lane, aligned4, w);  // in flight while the table is made

    TableLds& L = *reinterpret_cast<TableLds*>(&S.stage[0][0]);  // shares LDS with the chunk images, not in use yet
    static_assert(sizeof(TableLds) <= sizeof(S.stage), "table scratch must fit the chunk images");
    if constexpr (MODE == kPackBuild) {
        sum_partials<256>(L, p.hist_parts, p.n_parts, p.bits);
        rank_symbols<256>(L, p.bits);
        if (wave == 0) {
            TableOut out;
            out.entry = S.tab;
            table_from_hist_any(L, lane, p.bits, out);
            if (lane == 0) {
                S.max_len = out.max_len;
                S.payload_bits = out.payload_bits;
            }
        }
        __syncthreads();
        if (blockIdx.x == 0) p.stream[kHeaderBytes + tid] = (uint8_t)(S.tab[tid] >> 56);  // the container's length table
    } else {
        S.tab[tid] = p.enc_table[tid];
        if (tid == 0) {
            // a static table does not know this tensor's bit count: it comes out of the look-back
            S.max_len = MODE == kPackStatic ? p.static_max_len : p.ctrl->max_len;
            S.payload_bits = MODE == kPackStatic ? 0ull : p.ctrl->payload_bits;
        }
        __syncthreads();
        if (MODE == kPackStatic && blockIdx.x == 0) p.stream[kHeaderBytes + tid] = (uint8_t)(S.tab[tid] >> 56);
    }
    // nobody reads the table scratch any more: the images start out clear
    pack_clear_image(S, wave, lane);
    pack_group<MODE>(S, p, group, w, chunk_len_of(p, group * kPackWaves + (uint32_t)wave), []() {});
}

// ---------------------------------------------------------------------------
// Large tensors (more chunk groups than the device holds pack workgroups): three kernels that
// never wait for one another inside a launch, so nothing depends on which workgroups are
// resident.  k_chunk_bits sums the code lengths of every chunk; k_chunk_scan (one workgroup)
// turns them into the container's chunk offsets and writes the header; k_pack_at packs every
// chunk at its known place.  The symbols are read twice (they were just written and mostly come
// from the memory-side cache); the table is read from memory (k_huffman_table or a fixed one).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_chunk_bits(PackParams p) {
    __shared__ uint8_t s_len[256];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t stride = gridDim.x * kPackWaves;
    uint32_t ch = blockIdx.x * kPackWaves + (uint32_t)wave;
    // (lanes with four neighbouring symbols each, as in the pack kernel: 16-byte loads per lane were tried for this
    // sum, where the order does not matter, and took 21 us against 12 us at 51 M symbols)
    const bool aligned4 = (p.chunk_syms & 3u) == 0;
    uint32_t w[16];
    if (ch < p.n_chunks) load_chunk_symbols(p, ch, lane, aligned4, w);  // in flight while the lengths arrive
    s_len[tid] = (uint8_t)(p.enc_table[tid] >> 56);
    __syncthreads();
    while (ch < p.n_chunks) {  // wavefront-uniform
        const uint32_t clen = chunk_len_of(p, ch);
        const uint32_t next = ch + stride;
        uint32_t wn[16];
        if (next < p.n_chunks) load_chunk_symbols(p, next, lane, aligned4, wn);
        uint32_t bits = 0;
        if (clen == 4096u) {
#pragma unroll
            for (int q = 0; q < 16; q++)
#pragma unroll
                for (int i = 0; i < 4; i++) bits += s_len[(w[q] >> (8 * i)) & 255u];
        } else if (clen >= 3840u) {
            // (whole chunks of channel counts that do not divide 4096 -- 4032 symbols at 144 channels, 3840 at 960:
            // fifteen whole registers in one straight run, the tests for the last one only)
#pragma unroll
            for (int q = 0; q < 15; q++)
#pragma unroll
                for (int i = 0; i < 4; i++) bits += s_len[(w[q] >> (8 * i)) & 255u];
#pragma unroll
            for (int i = 0; i < 4; i++)
                if (3840u + 4u * (uint32_t)lane + i < clen) bits += s_len[(w[15] >> (8 * i)) & 255u];
        } else {
            // registers that lie inside the chunk whole need no per-symbol test
#pragma unroll
            for (int q = 0; q < 16; q++) {
                if (256u * (q + 1) <= clen) {  // wavefront-uniform
#pragma unroll
                    for (int i = 0; i < 4; i++) bits += s_len[(w[q] >> (8 * i)) & 255u];
                } else {
#pragma unroll
                    for (int i = 0; i < 4; i++)
                        if (256u * q + 4u * (uint32_t)lane + i < clen) bits += s_len[(w[q] >> (8 * i)) & 255u];
                }
            }
        }
        bits = wave_sum(bits);
        if (lane == 0) p.chunk_bits[ch] = bits;
        ch = next;
#pragma unroll
        for (int q = 0; q < 16; q++) w[q] = wn[q];
    }
}

// One workgroup: chunk_off[i] = words of the chunks before chunk i (a chunk starts on a word), the header, the
// stream size and the zero bytes of the alignment gaps.  The stream is marked invalid if it would outgrow the buffer.
// Rounds of kScanTile chunks: a thread takes kScanPer neighbouring entries (16-byte loads, all in flight together;
// the array's allocation is a multiple of 256 bytes, so a piece that starts inside it ends inside it), scans them in
// registers, the threads' sums are scanned across the workgroup, and the offsets leave as 16-byte stores (the offset
// table starts 320 bytes into the container, itself 16-byte aligned).
constexpr int kScanThreads = 1024, kScanPer = 16, kScanTile = kScanThreads * kScanPer;
__global__ __launch_bounds__(kScanThreads) void k_chunk_scan(PackParams p) {
    __shared__ unsigned long long s_wave[2][kScanThreads / 64];
    __shared__ unsigned long long s_bits[kScanThreads / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t n = p.n_chunks;
    uint32_t* chunk_off = reinterpret_cast<uint32_t*>(p.stream + kHeaderBytes + kLenTableBytes);
    unsigned long long carry = 0, bits = 0;
    int flip = 0;
    for (uint32_t base = 0; base < n; base += kScanTile, flip ^= 1) {
        const uint32_t i0 = base + (uint32_t)tid * kScanPer;
        uint32_t v[kScanPer];
#pragma unroll
        for (int k = 0; k < kScanPer; k += 4) {
            uint4 q = make_uint4(0u, 0u, 0u, 0u);
            if (i0 + k < n) q = *reinterpret_cast<const uint4*>(p.chunk_bits + i0 + k);
            v[k] = q.x; v[k + 1] = q.y; v[k + 2] = q.z; v[k + 3] = q.w;
        }
        uint32_t sum = 0;
#pragma unroll
        for (int k = 0; k < kScanPer; k++) {
            if (i0 + k >= n) v[k] = 0u;  // past the last chunk: whatever the workspace holds there
            bits += v[k];
            v[k] = (v[k] + 31u) >> 5;
            sum += v[k];
        }
        const unsigned long long incl = wave_inclusive_scan64(sum, lane);
        if (lane == 63) s_wave[flip][wave] = incl;
        __syncthreads();  // (the other buffer is what the round before used: no second barrier needed)
        unsigned long long before = carry + incl - sum, total = 0;
        for (int q = 0; q < kScanThreads / 64; q++) {
            if (q < wave) before += s_wave[flip][q];
            total += s_wave[flip][q];
        }
        uint32_t off[kScanPer];
#pragma unroll
        for (int k = 0; k < kScanPer; k++) {
            off[k] = (uint32_t)before;
            before += v[k];
        }
#pragma unroll
        for (int k = 0; k < kScanPer; k += 4) {
            if (i0 + k + 3 < n) {
                *reinterpret_cast<uint4*>(chunk_off + i0 + k) = make_uint4(off[k], off[k + 1], off[k + 2], off[k + 3]);
            } else {
#pragma unroll
                for (int j = 0; j < 4; j++)
                    if (i0 + k + j < n) chunk_off[i0 + k + j] = off[k + j];
            }
        }
        carry += total;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) bits += __shfl_xor(bits, o, 64);
    if (lane == 0) s_bits[wave] = bits;
    __syncthreads();
    if (tid == 0) {
        const unsigned long long total_words = carry;
        unsigned long long total_bits = 0;
        for (int q = 0; q < kScanThreads / 64; q++) total_bits += s_bits[q];
        chunk_off[n] = (uint32_t)total_words;
        Header hdr = p.hdr;
        hdr.payload_words = total_words;
        hdr.payload_bits = total_bits;
        if (total_words > p.cap_words || total_words > 0xffffffffull) hdr.magic = 0u;  // does not fit: not valid
        *reinterpret_cast<Header*>(p.stream) = hdr;
        if (p.out_bytes) *p.out_bytes = (uint64_t)p.off_payload + 4 * total_words;
        // alignment gaps between the sections are part of the stream: keep them zero
        for (size_t o = kHeaderBytes + kLenTableBytes + 4 * ((size_t)n + 1); o < p.off_sub_bits; o++) p.stream[o] = 0;
        for (size_t o = p.off_sub_bits + 2 * (size_t)n * p.subs_per_chunk; o < p.off_payload; o++) p.stream[o] = 0;
    }
}

// Packs every chunk at the place k_chunk_scan gave it.  One wavefront per chunk and turn, no barriers after the
// table is in LDS, the next chunk's symbols in flight while this one is packed.  STATIC: the table is a fixed one
// (its longest code comes with the parameters, and the block that holds chunk 0 writes the container's length
// table); otherwise k_huffman_table has left both.
template <bool STATIC>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 4))) void k_pack_at(PackParams p) {
    __shared__ PackShared S;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool aligned4 = (p.chunk_syms & 3u) == 0;
    uint32_t ch = blockIdx.x * kPackWaves + (uint32_t)wave;
    uint32_t w[16];
    if (ch < p.n_chunks) load_chunk_symbols(p, ch, lane, aligned4, w);
    S.tab[tid] = p.enc_table[tid];
    if (STATIC && blockIdx.x == 0) p.stream[kHeaderBytes + tid] = (uint8_t)(p.enc_table[tid] >> 56);
    pack_clear_image(S, wave, lane);
    __syncthreads();
    const uint32_t max_len = STATIC ? p.static_max_len : p.ctrl->max_len;
    uint32_t* img = S.stage[wave];
    uint16_t* sub_bits = reinterpret_cast<uint16_t*>(p.stream + p.off_sub_bits);
    const uint32_t* chunk_off = reinterpret_cast<const uint32_t*>(p.stream + kHeaderBytes + kLenTableBytes);
    uint32_t* payload = reinterpret_cast<uint32_t*>(p.stream + p.off_payload);
    const uint32_t n_runs = p.subs_per_chunk;
    auto sync_wave = [&]() {
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    };
    while (ch < p.n_chunks) {  // wavefront-uniform
        const uint32_t clen = chunk_len_of(p, ch);
        const uint32_t next = ch + gridDim.x * kPackWaves;
        uint32_t wn[16];
        if (next < p.n_chunks) load_chunk_symbols(p, next, lane, aligned4, wn);
        const uint32_t word0 = chunk_off[ch], word1 = chunk_off[ch + 1];
        auto build_window = [&](uint32_t win, uint32_t win_words, uint16_t* run_bits) -> uint32_t {
            uint32_t total;
            if (win == 0) {
                if (max_len <= 32) total = pack_chunk<false, true>(w, clen, S.tab, img, win, win_words, lane, run_bits, n_runs);
                else total = pack_chunk<true, true>(w, clen, S.tab, img, win, win_words, lane, run_bits, n_runs);
            } else {
                if (max_len <= 32) total = pack_chunk<false, false>(w, clen, S.tab, img, win, win_words, lane, run_bits, n_runs);
                else total = pack_chunk<true, false>(w, clen, S.tab, img, win, win_words, lane, run_bits, n_runs);
            }
            sync_wave();  // the ORs of all lanes precede the reads that follow
            return total;
        };
        uint16_t* runs_out = sub_bits + (size_t)ch * n_runs;
        const bool staged = n_runs <= 64u;
        const uint32_t total_bits = build_window(0, kStageWords, staged ? S.runs[wave] : runs_out);
        if (staged && (uint32_t)lane < n_runs) runs_out[lane] = S.runs[wave][lane];
        const uint32_t n_words = (total_bits + 31) >> 5;
        // what the size pass counted must be what this pass produces (the same symbols and table); should the
        // symbols have changed in between, or the payload not fit, nothing is written past the chunk's place and
        // the stream is left invalid
        const bool fits = word1 - word0 == n_words && (uint64_t)word0 + n_words <= p.cap_words;
        if (!fits && lane == 0) *reinterpret_cast<uint32_t*>(p.stream) = 0u;  // the header's magic
        for (uint32_t win = 0; win < n_words; win += kStageWords) {
            const uint32_t win_words = (n_words - win < (uint32_t)kStageWords) ? n_words - win : (uint32_t)kStageWords;
            if (win) build_window(win, win_words, nullptr);
            for (uint32_t i = lane; i < win_words; i += 64) {
                if (fits) payload[(size_t)word0 + win + i] = img[i];
                img[i] = 0u;
            }
            sync_wave();  // the image is read and clear before the next window or chunk writes it
        }
        ch = next;
#pragma unroll
        for (int q = 0; q < 16; q++) w[q] = wn[q];
    }
}

// Number of workgroups of the pack kernel the device holds at once (queried once per kernel variant).
template <int MODE>
static int pack_resident_groups() {
    static std::atomic<int> cached{0};  // (every thread computes the same value)
    if (int c = cached.load(std::memory_order_relaxed)) return c;
    int dev = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_pack<MODE>, 256, 0) != hipSuccess || cus < 1 ||
        per_cu < 1)
        return 64;  // conservative: any device this library runs on holds 64 workgroups
    if (per_cu > 4) per_cu = 4;
    cached.store(cus * per_cu, std::memory_order_relaxed);
    return cus * per_cu;
}

// Table (a kernel of its own only where every pack workgroup building it would cost more than the launch)
// and packing.
PackParams pack_params(const uint8_t* d_syms, const Geometry& g, int bits, float delta, const CoderScratch& cs,
                       int n_parts, const uint64_t* d_enc_table, uint8_t* d_stream, uint64_t cap_words,
                       uint64_t* d_out_bytes) {
    PackParams p{};
    p.cap_words = cap_words;
    p.syms = d_syms;
    p.V = (uint64_t)g.P * (uint64_t)g.C;
    p.n_chunks = g.n_chunks;
    p.chunk_syms = g.chunk_syms;
    p.subs_per_chunk = g.subs_per_chunk;
    p.n_groups = cs.n_groups;
    p.chunk_bits = cs.chunk_bits;
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

// Sizes, offsets and packing of a tensor with more chunk groups than the device holds pack workgroups.
template <bool STATIC>
static hipError_t launch_pack_large(const PackParams& p, hipStream_t s) {
    if (!p.chunk_bits) return hipErrorInvalidValue;
    const uint32_t n_groups = pack_groups(p.n_chunks);
    const uint32_t cap = (uint32_t)pack_resident_groups<kPackTable>();
    const uint32_t grid = n_groups < 2 * cap ? n_groups : 2 * cap;
    hipError_t e = launch(K_CHUNK_BITS, k_chunk_bits, dim3(grid), dim3(256), 0, s, p);
    if (e != hipSuccess) return e;
    e = launch(K_CHUNK_SCAN, k_chunk_scan, dim3(1), dim3(kScanThreads), 0, s, p);
    if (e != hipSuccess) return e;
    return launch(K_PACK, k_pack_at<STATIC>, dim3(n_groups < cap ? n_groups : cap), dim3(256), 0, s, p);
}

hipError_t launch_coder(const uint8_t* d_syms, const Geometry& g, int bits, float delta, const CoderScratch& cs,
                        int n_parts, uint64_t* d_enc_table, uint8_t* d_stream, uint64_t cap_words,
                        uint64_t* d_out_bytes, hipStream_t s) {
    PackParams p = pack_params(d_syms, g, bits, delta, cs, n_parts, d_enc_table, d_stream, cap_words, d_out_bytes);
    const uint32_t resident = (uint32_t)pack_resident_groups<kPackTable>();
    const bool large = cs.n_groups > resident;
    // every pack workgroup sums the partial histograms itself while that is at most 64 KB to read
    const bool build_in_pack = !large && ((size_t)n_parts << bits) * 4 <= 64 * 1024;
    if (!build_in_pack) {
        hipError_t e = launch(K_TABLE, k_huffman_table, dim3(1), dim3(1024), 0, s, (const uint32_t*)cs.hist_parts,
                              n_parts, bits, (uint32_t*)nullptr, d_enc_table, d_stream + kHeaderBytes, cs.ctrl, 0u);
        if (e != hipSuccess) return e;
        if (large) return launch_pack_large<false>(p, s);
        return launch(K_PACK, k_pack<kPackTable>, dim3(cs.n_groups), dim3(256), 0, s, p);
    }
    const uint32_t cap = (uint32_t)pack_resident_groups<kPackBuild>();
    if (cs.n_groups > cap) return hipErrorInvalidValue;  // (not reachable: the two variants hold the same number)
    return launch(K_PACK, k_pack<kPackBuild>, dim3(cs.n_groups), dim3(256), 0, s, p);
}

// Packing with a table fixed beforehand (one code for every symbol of the alphabet): no histogram, no table build.
// The coder's counters must be clear (the kernel that made the symbols clears them).
hipError_t launch_coder_static(const uint8_t* d_syms, const Geometry& g, int bits, float delta, const CoderScratch& cs,
                               const uint64_t* d_enc_table, uint32_t max_len, uint8_t* d_stream, uint64_t cap_words,
                               uint64_t* d_out_bytes, hipStream_t s) {
    PackParams p = pack_params(d_syms, g, bits, delta, cs, 0, d_enc_table, d_stream, cap_words, d_out_bytes);
    p.static_max_len = max_len;
    const uint32_t cap = (uint32_t)pack_resident_groups<kPackStatic>();
    if (cs.n_groups > cap) return launch_pack_large<true>(p, s);
    return launch(K_PACK, k_pack<kPackStatic>, dim3(cs.n_groups), dim3(256), 0, s, p);
}

}  // namespace fmtc
