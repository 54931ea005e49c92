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
    if (tid < 256) L.h[tid] = 0u;
    __syncthreads();
    // a thread owns four neighbouring bins of every rstep-th row; eight independent 16-byte loads in flight
    const int tpr = K / 4, col = tid % tpr, row0 = tid / tpr, rstep = THREADS / tpr;
    const uint4* rows = reinterpret_cast<const uint4*>(hist_parts);
    uint4 acc = make_uint4(0, 0, 0, 0);
    int q = row0;
    for (; q + 7 * rstep < n_parts; q += 8 * rstep) {
        uint4 v[8];
#pragma unroll
        for (int j = 0; j < 8; j++) v[j] = rows[(size_t)(q + j * rstep) * tpr + col];
#pragma unroll
        for (int j = 0; j < 8; j++) {
            acc.x += v[j].x; acc.y += v[j].y; acc.z += v[j].z; acc.w += v[j].w;
        }
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

// What the table build leaves for its caller.
struct TableOut {
    unsigned long long* entry;  // [256] (LDS): bit-reversed code | length << 56
    uint32_t max_len;
    unsigned long long payload_bits;
};

// Code table from the histogram L.h.  Runs in ONE wavefront (64 lanes, `lane`), no workgroup barrier inside;
// lane l owns symbols l, l + 64, ... (NVS = alphabet size / 64, at least 1).  Every lane returns the same
// max_len and payload_bits; entry[] is complete when the function returns (for this wavefront).
template <int NVS>
__device__ __forceinline__ void table_from_hist(TableLds& L, int lane, int K, TableOut& out) {
    uint32_t cnt[NVS], rank[NVS];
#pragma unroll
    for (int j = 0; j < NVS; j++) {
        cnt[j] = (64 * j + lane < K) ? L.h[64 * j + lane] : 0u;
        rank[j] = 0;
    }
    // position of every used symbol in (count, symbol) order (K is a multiple of 4: four counts per LDS read)
    for (int t = 0; t < K; t += 4) {
        const uint4 o4 = *reinterpret_cast<const uint4*>(&L.h[t]);
        const uint32_t o[4] = {o4.x, o4.y, o4.z, o4.w};
#pragma unroll
        for (int i = 0; i < 4; i++)
#pragma unroll
            for (int j = 0; j < NVS; j++)
                rank[j] += (o[i] != 0 && (o[i] < cnt[j] || (o[i] == cnt[j] && t + i < 64 * j + lane))) ? 1u : 0u;
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
    uint32_t len[NVS], before[NVS];
    uint32_t max_len = 0;
    unsigned long long pbits = 0;
#pragma unroll
    for (int j = 0; j < NVS; j++) {
        len[j] = cnt[j] ? (uint32_t)L.len_sorted[rank[j]] : 0u;
        before[j] = 0;
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
    // codes of one length are numbered in symbol order; lane q ends up with the number of codes of length q
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
        out.entry[64 * j + lane] = entry;
    }
    if (NVS < 4)
        for (int s = 64 * NVS + lane; s < 256; s += 64) out.entry[s] = 0ull;
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
                                                        CoderCtrl* __restrict__ ctrl) {
    __shared__ TableLds L;
    __shared__ unsigned long long entry[256];
    sum_partials<1024>(L, hist_parts, n_parts, bits);
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

// Appends the codes of one run (`cnt` symbols, 64 at most, four per register of w) to the image, starting at
// bit `start` of the chunk.  FULL: cnt == 64.  LONG: codes may exceed 32 bits.
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
        for (int q = 0; q < 16; q++) {
            // the four table reads do not depend on the bit position: they are in flight together
            unsigned long long e[4];
#pragma unroll
            for (int b = 0; b < 4; b++) e[b] = tab[(w[q] >> (8 * b)) & 255u];
#pragma unroll
            for (int b = 0; b < 4; b++) {
                if (FULL || (uint32_t)(4 * q + b) < cnt) {
                    const uint32_t code = (uint32_t)e[b], len = (uint32_t)(e[b] >> 56);
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

// kPackWaves chunks per workgroup: one wavefront per chunk, one lane per run of 64 symbols.
template <bool BUILD>
__global__ __launch_bounds__(256) void k_pack(PackParams p) {
    static_assert(kPackWaves == 4, "one chunk per wavefront of the 256-thread workgroup");
    __shared__ unsigned long long tab[256];
    __shared__ __align__(16) uint32_t stage[kPackWaves][kStageWords];
    __shared__ uint32_t wave_words[kPackWaves];
    __shared__ uint32_t s_group, s_excl, s_max_len;
    __shared__ unsigned long long s_payload_bits;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wavefront-uniform by construction
    if (tid == 0) s_group = __hip_atomic_fetch_add(&p.ctrl->ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    TableLds& L = *reinterpret_cast<TableLds*>(&stage[0][0]);  // shares LDS with the chunk images, not in use yet
    static_assert(sizeof(TableLds) <= sizeof(stage), "table scratch must fit the chunk images");
    if constexpr (BUILD) {
        sum_partials<256>(L, p.hist_parts, p.n_parts, p.bits);
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

    // ---- the run: 64 symbols in 16 registers (the loads are in flight while wavefront 0 builds the table) ----
    uint32_t w[16];
#pragma unroll
    for (int q = 0; q < 16; q++) w[q] = 0;
    uint32_t cnt = 0;
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
    }
    if constexpr (BUILD) {
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
        if (group == 0) p.stream[kHeaderBytes + tid] = (uint8_t)(tab[tid] >> 56);  // the container's length table
    }
    const bool long_codes = s_max_len > 32;
    const bool all_full = __all(cnt == (uint32_t)kSubSyms || cnt == 0u) != 0;

    // ---- pass 1: code bits of the run ----
    uint32_t bits = 0;
    if (all_full) {
        if (cnt) {
            uint32_t part[4] = {0u, 0u, 0u, 0u};  // four independent sums
#pragma unroll
            for (int q = 0; q < 16; q++)
#pragma unroll
                for (int b = 0; b < 4; b++) part[b] += (uint32_t)(tab[(w[q] >> (8 * b)) & 255u] >> 56);
            bits = (part[0] + part[1]) + (part[2] + part[3]);
        }
    } else {
#pragma unroll
        for (int q = 0; q < 16; q++)
#pragma unroll
            for (int b = 0; b < 4; b++)
                if ((uint32_t)(4 * q + b) < cnt) bits += (uint32_t)(tab[(w[q] >> (8 * b)) & 255u] >> 56);
    }
    if (have) {
        uint16_t* sub_bits = reinterpret_cast<uint16_t*>(p.stream + p.off_sub_bits);
        if ((uint32_t)lane < p.subs_per_chunk) sub_bits[(size_t)ch * p.subs_per_chunk + lane] = (uint16_t)bits;
    }
    const uint32_t start = wave_exclusive_scan(bits, lane);
    const uint32_t total_bits = __shfl(start + bits, 63, 64);
    const uint32_t n_words = (total_bits + 31) >> 5;
    if (lane == 0) wave_words[wave] = n_words;
    __syncthreads();  // also: nobody reads the table scratch any more, the images may be written
    uint32_t agg = 0;
#pragma unroll
    for (int q = 0; q < kPackWaves; q++) agg += wave_words[q];
    if (tid == 0) publish64(&p.lookback[group], (group == 0 ? kFlagInclusive : kFlagAggregate) | agg);

    // ---- pass 2 for the first window: needs no global position, so it runs while the predecessors publish ----
    uint32_t* img = stage[wave];
    const uint32_t first_word = start >> 5, last_word = (start + bits + 31) >> 5;  // [first, last)
    auto build_window = [&](uint32_t win, uint32_t win_words) {
        for (uint32_t i = lane; i < win_words; i += 64) img[i] = 0u;
        wave_sync();  // the zeros land before the ORs below: one wavefront, LDS in order
        if (cnt && bits && first_word < win + win_words && last_word > win) {
            if (long_codes) pack_run<false, true>(w, cnt, start, tab, img, win, win_words);
            else if (all_full) pack_run<true, false>(w, cnt, start, tab, img, win, win_words);
            else pack_run<false, false>(w, cnt, start, tab, img, win, win_words);
        }
        wave_sync();  // the ORs of all lanes precede the reads that follow
    };
    const uint32_t win0_words = n_words < (uint32_t)kStageWords ? n_words : (uint32_t)kStageWords;
    if (have && n_words) build_window(0, win0_words);

    // ---- the group's first payload word: the words of all groups before it ----
    if (wave == 0 && group != 0) {
        // windows of 256 predecessors, nearest first; lane l reads four of them
        uint32_t excl = 0;
        uint32_t top = group;  // predecessors [0, top) are still to be accounted for
        bool failed = false;
        while (top > 0) {
            uint32_t sum = 0;
            bool found = false;  // met a running total: everything before it is included
            bool ready = false;
            for (uint32_t tries = 0; tries < kSpinLimit; tries++) {
                unsigned long long e[4];
#pragma unroll
                for (int j = 0; j < 4; j++) {
                    const uint32_t back = 4u * (uint32_t)lane + (uint32_t)j + 1u;  // distance to the predecessor
                    e[j] = (back <= top) ? peek64(&p.lookback[top - back]) : kFlagAggregate;
                }
                sum = 0;
                found = false;
                bool ok = true;
#pragma unroll
                for (int j = 0; j < 4; j++) {
                    if (!found) {
                        if (e[j] == 0) ok = false;
                        sum += (uint32_t)e[j];
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
            const uint32_t part = (lane <= first) ? sum : 0u;
            excl += wave_sum(part);
            if (fmask) break;
            top = (top > 256u) ? top - 256u : 0u;
        }
        if (failed) {
            if (lane == 0) p.ctrl->error = 1u;
            excl = 0;
        }
        if (lane == 0) {
            publish64(&p.lookback[group], kFlagInclusive | (unsigned long long)(excl + agg));
            s_excl = excl;
        }
    } else if (tid == 0) {
        s_excl = 0;
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

    // ---- the image leaves with full-width stores; further windows (rare) are built and stored in turn ----
    uint32_t* out = reinterpret_cast<uint32_t*>(p.stream + p.off_payload) + word0;
    for (uint32_t win = 0; win < n_words; win += kStageWords) {
        const uint32_t win_words = (n_words - win < (uint32_t)kStageWords) ? n_words - win : (uint32_t)kStageWords;
        if (win) build_window(win, win_words);
        for (uint32_t i = lane; i < win_words; i += 64) out[win + i] = img[i];
        wave_sync();  // all lanes have read the image before the next window clears it
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
