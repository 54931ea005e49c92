// Decoder (paper section 3: variable length decoder, inverse quantizer, inverse
// transform; section 3.1 "Implementation": levels scaled back to the transform
// domain, then the inverse PCA).  One kernel per call:
//   1. every workgroup checks the header and the code length table and builds the
//      canonical decode tables and a 2^11-entry three-symbol lookup table in LDS;
//   2. one wavefront per chunk, one lane per run of 64 symbols (bit offset = prefix
//      sum of the stored run sizes) decodes into an LDS symbol tile;
//   3. x_hat = T^T (Delta q) + mu on the f16 matrix cores
//      (v_mfma_f32_32x32x16_f16; the levels are exact in f16, the basis entries are
//      split in two f16 parts).  Narrow tensors (up to 160 channels): the wavefront
//      that decoded a chunk also transforms it, the basis sits in LDS in operand
//      order and no workgroup barrier is needed after the tables.  Wide tensors: a
//      tile of several chunks per workgroup, the basis streamed from L2.
// Nothing outside [stream, stream + bytes) is read whatever the stream holds.
#include "fmtc_device.h"
#include "fmtc_internal.h"

namespace fmtc {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));
typedef _Float16 halfx2 __attribute__((ext_vector_type(2)));

// byte address of symbol n of the tile: every run of 64 symbols is followed by 4
// pad bytes so that the 64 lanes of a decoding wavefront hit different banks
__device__ __forceinline__ uint32_t sym_addr(uint32_t n) { return n + 4u * (n >> 6); }


constexpr int kLut2Bits = 10;  // second table: codes longer than kLutBits bits

// Where the lookup table keeps the entry of the stream bits `v` (kLutBits of them, first bit lowest).  The LDS bank of
// a word is its index modulo 64; short codes are frequent, so many lanes of a wavefront look at bit patterns that
// agree in their first bits and differ in the later ones -- with the plain index these would be different words of
// one bank, read one after the other.  Folding the upper bits into the lower six spreads them over the banks
// (patterns that agree in all bits are one word, which the LDS reads once for all lanes).
__device__ __forceinline__ uint32_t lut_slot(uint32_t v) { return v ^ (v >> 6); }
// The same for the 16-bit scratch table of the construction (two entries per word: bits 1..6 choose the bank), which
// is read at values shifted left by a code length: their lower bits are zero, and the upper ones must choose the bank.
__device__ __forceinline__ uint32_t first_slot(uint32_t v) { return v ^ (v >> 5); }

// Decode tables, in LDS, built by every workgroup from the code length table of the stream.
struct DecTables {
    uint32_t cnt_len[64];     // number of codes of each length
    uint32_t first_rank[64];  // rank (in (length, symbol) order) of the first code of each length
    uint64_t first_code[64];  // first canonical code of each length
    uint64_t limit[64];       // (first_code + count) << (32 - length) for length <= 32: first left-aligned 32-bit
                              // value that is NOT a code of this length or shorter
    uint32_t limit32[64];     // the same, saturated to 32 bits (exact for every length below the longest)
    uint16_t sorted_sym[256]; // symbols in (length, symbol) order
    // next kLutBits stream bits -> up to three symbols: sym0 | sym1 << 8 | sym2 << 16 | bits << 24 | n << 29,
    // n = number of whole codes found in those bits (0: the first code is longer than kLutBits), bits = their
    // total length
    uint32_t lut[1 << kLutBits];
    // Codes longer than kLutBits bits.  Canonical codes grow with their length, so left-aligned in 32 bits all of
    // them lie at or above long_base (the first value the short codes do not cover), in a range whose size is about
    // their share of the probability mass.  lut2 is indexed by (value - long_base) >> long_shift: sym | len << 8
    // where those bits decide the code (its length is at most 32 - long_shift and at most 31), 0 where they do not
    // (the decoders then search the per-length limits).  It shares its place with scratch of the construction:
    // `first` = first code in a kLutBits-bit value (first stream bit on top), sym | len << 8.
    union {
        uint16_t lut2[1 << kLut2Bits];
        uint16_t first[1 << kLutBits];
    };
    uint32_t wave_len_count[4][64];
    uint32_t lut_limit[kLutBits + 1];  // limit[] in a kLutBits-bit frame
    uint32_t n_used, bad_len, ok, max_len;
    uint32_t long_base, long_shift, pad0, pad1;
};

// All THREADS threads of the workgroup call this (THREADS a multiple of 256); my_len is the code length of symbol
// threadIdx.x from the stream (threads past 255: anything).  Returns false (for every thread)
// unless the lengths form a complete prefix code (Kraft sum exactly 1), or the single one-bit code of a
// one-symbol tensor.
template <int THREADS>
__device__ __forceinline__ bool build_decode_tables(DecTables& T, int my_len, int bits) {
    const int tid = threadIdx.x, lane = tid & 63;
    const int K = 1 << bits;
    if (tid < 64) T.cnt_len[tid] = 0u;
    if (tid < 256) T.wave_len_count[tid >> 6][tid & 63] = 0u;
    if (tid == 0) { T.n_used = 0u; T.bad_len = 0u; }
    __syncthreads();
    if (tid < 256) {
        if (my_len > kMaxLen || (tid >= K && my_len != 0)) {
            atomicAdd(&T.bad_len, 1u);
            my_len = 0;
        } else if (my_len) {
            atomicAdd(&T.cnt_len[my_len], 1u);
            atomicAdd(&T.n_used, 1u);
        }
    }
    __syncthreads();
    if (tid < 64) {
        // running sums over the lengths: count(j) * 2^(48-j) gives the first code of each length (shifted down to
        // its own width), the Kraft sum and the "first value that is no code of this length" limits
        const bool in = tid >= 1 && tid <= kMaxLen;
        const uint32_t c = in ? T.cnt_len[tid] : 0u;
        const unsigned long long w = (unsigned long long)c << (in ? kMaxLen - tid : 0);
        const unsigned long long incl = wave_inclusive_scan64(w, lane);
        const uint32_t rank = wave_exclusive_scan(c, lane);
        const unsigned long long kraft = __shfl(incl, 63, 64);
        T.first_code[tid] = in ? ((incl - w) >> (kMaxLen - tid)) : 0ull;
        T.first_rank[tid] = in ? rank : 0u;
        const unsigned long long lim32 = (in && tid <= 32) ? (incl >> (kMaxLen - 32)) : ~0ull;
        T.limit[tid] = lim32;
        T.limit32[tid] = lim32 > 0xffffffffull ? 0xffffffffu : (uint32_t)lim32;
        if (tid >= 1 && tid <= kLutBits) T.lut_limit[tid] = (uint32_t)(incl >> (kMaxLen - kLutBits));
        if (!in) T.cnt_len[tid] = 0u;
        const unsigned long long used = __ballot(c != 0);
        if (tid == 0) {
            const uint32_t n = T.n_used;
            T.max_len = used ? (uint32_t)(63 - __clzll((long long)used)) : 0u;
            T.ok = (T.bad_len == 0 && n >= 1 && (n == 1 ? T.cnt_len[1] == 1 : kraft == (1ull << kMaxLen))) ? 1u : 0u;
        }
    }
    __syncthreads();
    if (!T.ok) return false;
    // symbols of equal length are numbered in symbol order
    uint32_t before = 0;
    if (tid < 256) {
        // the lanes of this wavefront with the same length as this one: six ballots, one per bit of the length
        unsigned long long same = ~0ull;
#pragma unroll
        for (int bit = 0; bit < 6; bit++) {
            const unsigned long long m = __ballot((my_len >> bit) & 1);
            same &= ((my_len >> bit) & 1) ? m : ~m;
        }
        before = (uint32_t)__popcll(same & ((1ull << lane) - 1ull));
        if (my_len && before == 0) T.wave_len_count[tid >> 6][my_len] = (uint32_t)__popcll(same);  // the first of them
    }
    __syncthreads();
    if (tid < 256) {
        if (my_len) {
            for (int q = 0; q < (tid >> 6); q++) before += T.wave_len_count[q][my_len];
            T.sorted_sym[T.first_rank[my_len] + before] = (uint16_t)tid;
        }
        if ((uint32_t)tid >= T.n_used) T.sorted_sym[tid] = 0;  // ranks past the last code stay harmless
    }
    __syncthreads();
    {
        // Step 1: the first code in every kLutBits-bit value.  Canonical codes, left-aligned, grow with their
        // length, so the length is 1 + the number of per-length limits the value reaches.  Fixed trip count,
        // unrolled: the searches of several values are independent and interleave.
        uint32_t lim[kLutBits + 1];
#pragma unroll
        for (int l = 1; l <= kLutBits; l++) lim[l] = T.lut_limit[l];
#pragma unroll
        for (int it = 0; it < ((1 << kLutBits) + THREADS - 1) / THREADS; it++) {
            const uint32_t v = (uint32_t)(tid + it * THREADS);
            // (only workgroup sizes that do not divide the table need the test: without it the turns are one
            // straight run and their dependent LDS reads overlap)
            if constexpr (((1 << kLutBits) % THREADS) != 0) {
                if (v >= (1u << kLutBits)) break;
            }
            uint32_t len = 1;
#pragma unroll
            for (int l = 1; l < kLutBits; l++) len += (v >= lim[l]) ? 1u : 0u;
            uint32_t entry = 0;
            if (v < lim[kLutBits]) {
                const uint32_t off = (v >> (kLutBits - len)) - (uint32_t)T.first_code[len];
                entry = (uint32_t)T.sorted_sym[(T.first_rank[len] + off) & 255u] | (len << 8);
            }
            T.first[first_slot(v)] = (uint16_t)entry;
        }
    }
    __syncthreads();
    {
        // Step 2: chain up to three codes per table entry (the index of an entry is in stream order, least
        // significant bit first).  A later code counts only if all its bits are inside the kLutBits bits.
        constexpr uint32_t kMask = (1u << kLutBits) - 1u;
#pragma unroll
        for (int it = 0; it < ((1 << kLutBits) + THREADS - 1) / THREADS; it++) {
            if constexpr (((1 << kLutBits) % THREADS) != 0) {
                if ((uint32_t)(tid + it * THREADS) >= (1u << kLutBits)) break;
            }
            // (neighbouring threads take neighbouring values v0: the reads of `first` below are neighbours, and the
            // entries, whose indices differ in their upper bits, go to different banks through lut_slot; taking
            // neighbouring indices instead puts every read of a wavefront on one bank)
            const uint32_t v0 = (uint32_t)(tid + it * THREADS);
            const int idx = (int)(__brev(v0) >> (32 - kLutBits));
            const uint32_t f0 = T.first[first_slot(v0)];
            const uint32_t len0 = f0 >> 8;
            const uint32_t v1 = (v0 << len0) & kMask;
            const uint32_t f1 = T.first[first_slot(v1)];
            const uint32_t len1 = f1 >> 8;
            const uint32_t v2 = (v1 << len1) & kMask;
            const uint32_t f2 = T.first[first_slot(v2)];
            const uint32_t len2 = f2 >> 8;
            const bool ok0 = len0 != 0;
            const bool ok1 = ok0 && len1 != 0 && len0 + len1 <= (uint32_t)kLutBits;
            const bool ok2 = ok1 && len2 != 0 && len0 + len1 + len2 <= (uint32_t)kLutBits;
            uint32_t e = 0;
            if (ok0) e = (f0 & 255u) | (len0 << 24) | (1u << 29);
            if (ok1) e = (f0 & 255u) | ((f1 & 255u) << 8) | ((len0 + len1) << 24) | (2u << 29);
            if (ok2) e = (f0 & 255u) | ((f1 & 255u) << 8) | ((f2 & 255u) << 16) | ((len0 + len1 + len2) << 24) | (3u << 29);
            T.lut[lut_slot((uint32_t)idx)] = e;
        }
    }
    __syncthreads();  // `first` is not read any more: the second table takes its place
    {
        // Step 3: the table of the longer codes (see DecTables).  Nothing to do where no code is longer than kLutBits.
        const uint32_t lim = T.lut_limit[kLutBits];  // kLutBits-bit values below it start with a short code
        const uint32_t max_len = T.max_len;
        const bool have_long = max_len > (uint32_t)kLutBits && lim < (1u << kLutBits);
        const uint32_t base = have_long ? lim << (32 - kLutBits) : 0xffffffffu;
        const uint64_t span = (1ull << 32) - base;  // values at or above base
        // the smallest shift that brings the span down to the table's 2^kLut2Bits entries (at most 32 - kLut2Bits),
        // in closed form: a loop over the candidates was 1.6 us of every workgroup's start
        uint32_t shift = 0;
        if (span > (1ull << kLut2Bits)) {
            const uint32_t m = 63u - (uint32_t)__clzll((long long)span);  // 2^m <= span < 2^(m+1), m > kLut2Bits - 1
            shift = m - kLut2Bits;
            if ((span >> shift) > (1ull << kLut2Bits)) shift++;
            if (shift > 32u - kLut2Bits) shift = 32u - kLut2Bits;
        }
        if (tid == 0) {
            T.long_base = base;
            T.long_shift = shift;
            T.pad0 = 0u;
            T.pad1 = 0u;
        }
        // (worth its construction only where long codes are frequent: their share of the code space, about their
        // share of the symbols, is span / 2^32; below 2^-11 a chunk meets a handful of them)
        if (have_long && span >= (1ull << 21)) {
            const uint32_t top = max_len < 33u ? max_len : 33u;
            uint32_t lim32[33 - (kLutBits + 1)];  // the limits, read once
#pragma unroll
            for (uint32_t l = kLutBits + 1; l < 33u; l++) lim32[l - (kLutBits + 1)] = T.limit32[l];
#pragma unroll
            for (int it = 0; it < ((1 << kLut2Bits) + THREADS - 1) / THREADS; it++) {
                const uint32_t idx = (uint32_t)tid + (uint32_t)(it * THREADS);
                if (idx >= (1u << kLut2Bits)) break;
                const uint64_t v64 = (uint64_t)base + ((uint64_t)idx << shift);
                const uint32_t v = (uint32_t)v64;
                uint32_t len = kLutBits + 1;
#pragma unroll
                for (uint32_t l = kLutBits + 1; l < 33u; l++) {
                    len += (l < top && v >= lim32[l - (kLutBits + 1)]) ? 1u : 0u;
                }
                uint32_t entry = 0;
                if (v64 <= 0xffffffffull && len <= 32u - shift && len <= 31u) {
                    const uint32_t off = (v >> (32 - len)) - (uint32_t)T.first_code[len];
                    if (off < T.cnt_len[len]) entry = (uint32_t)T.sorted_sym[(T.first_rank[len] + off) & 255u] | (len << 8);
                }
                T.lut2[idx] = (uint16_t)entry;
            }
        } else {
            // no entry of the first table sends a valid stream here; a corrupt one finds "undecided" and is caught
            // by the search
            for (uint32_t idx = (uint32_t)tid; idx < (1u << kLut2Bits); idx += THREADS) T.lut2[idx] = 0;
        }
    }
    __syncthreads();
    return true;
}

// Decode tables made once for a code table that is fixed beforehand, in global memory: what build_decode_tables
// leaves in LDS, and the code lengths they were made from.
struct PrebuiltTables {
    DecTables T;
    uint8_t len[256];
};
static_assert(sizeof(DecTables) % 16 == 0, "copied 16 bytes at a time");

// The prebuilt tables into LDS in place of building them -- after checking that the stream carries the very
// lengths they were made from (my_len: the stream's length of symbol threadIdx.x, threads past 255: anything).
// All THREADS threads call it; returns false for every thread on a mismatch.
template <int THREADS>
__device__ __forceinline__ bool load_decode_tables(DecTables& T, int my_len, const PrebuiltTables* pre) {
    const int tid = threadIdx.x;
    const uint4* src = reinterpret_cast<const uint4*>(&pre->T);
    uint4* dst = reinterpret_cast<uint4*>(&T);
    for (int i = tid; i < (int)(sizeof(DecTables) / 16); i += THREADS) dst[i] = src[i];
    const int mismatch = (tid < 256 && my_len != (int)pre->len[tid]) ? 1 : 0;
    return __syncthreads_or(mismatch) == 0;  // (also the barrier behind the copy)
}

__global__ __launch_bounds__(256) void k_build_decode_tables(const uint8_t* __restrict__ len_table, int bits,
                                                             PrebuiltTables* __restrict__ out, uint32_t* __restrict__ ok) {
    __shared__ __align__(16) DecTables T;
    const int tid = threadIdx.x;
    const bool good = build_decode_tables<256>(T, (int)len_table[tid], bits);
    if (tid == 0) *ok = good ? 1u : 0u;
    if (!good) return;
    const uint4* src = reinterpret_cast<const uint4*>(&T);
    uint4* dst = reinterpret_cast<uint4*>(&out->T);
    for (int i = tid; i < (int)(sizeof(DecTables) / 16); i += 256) dst[i] = src[i];
    out->len[tid] = len_table[tid];
}

hipError_t launch_build_decode_tables(const uint8_t* d_len_table, int bits, void* d_prebuilt, uint32_t* d_ok, hipStream_t s) {
    return launch(K_TABLE, k_build_decode_tables, dim3(1), dim3(256), 0, s, d_len_table, bits,
                  static_cast<PrebuiltTables*>(d_prebuilt), d_ok);
}
size_t prebuilt_decode_tables_bytes() { return sizeof(PrebuiltTables); }

// Decodes the `cnt` symbols of one run (one lane) starting at bit `start` of a chunk into the symbol tile.
// STAGED: the chunk's words are in LDS (`pw`, two zero words behind them); otherwise they are read from
// global memory (`gw`), zero past the chunk's end.  Returns false if bits matched no code word.
// State: lo/hi are payload words widx and widx+1, sh the bit offset in lo, nxt word widx+2 (read ahead),
// so 32 valid bits are at hand for every table lookup and a step crosses at most one word boundary.
//
// Output of a run: symbol n of the tile at sym_addr(n).
struct ByteOut {
    uint8_t* tile;
    uint32_t a0, o, i;
    __device__ __forceinline__ ByteOut(uint8_t* t, uint32_t nbase) : tile(t), a0(nbase + 4u * (nbase >> 6)), o(nbase & 63u), i(0) {}
    __device__ __forceinline__ void put(uint32_t sym) {  // sym_addr(nbase + i) = a0 + i + 4 * ((o + i) >> 6)
        tile[a0 + i + (((o + i) >> 6) << 2)] = (uint8_t)sym;
        i++;
    }
};
template <bool STAGED, typename Out>
__device__ __forceinline__ bool decode_run(const uint32_t* pw, const uint32_t* __restrict__ gw, uint32_t nwords,
                                           uint32_t start, uint32_t cnt, const DecTables& T, Out out) {
    auto fetch = [&](uint32_t rel) -> uint32_t {
        if constexpr (STAGED) return pw[rel < nwords + 1 ? rel : nwords + 1];
        else return (rel < nwords) ? gw[rel] : 0u;
    };
    // word index can not wrap: start <= 64 runs * 65535 bits
    uint32_t widx = start >> 5, sh = start & 31;
    uint32_t lo = fetch(widx), hi = fetch(widx + 1), nxt = fetch(widx + 2);
    bool ok = true;
    uint32_t i = 0;
    while (i < cnt) {
        const uint32_t w = __builtin_amdgcn_alignbit(hi, lo, sh);
        uint32_t e = T.lut[lut_slot(w & ((1u << kLutBits) - 1))];
        uint32_t n = e >> 29, sym0 = e & 255u, len0 = (e >> 24) & 31u;
        if (n == 0) {  // a code longer than the table: the second table decides most of them
            const uint32_t e2 = T.lut2[((__brev(w) - T.long_base) >> T.long_shift) & ((1u << kLut2Bits) - 1)];
            if (e2) {
                sym0 = e2 & 255u;
                len0 = e2 >> 8;
                n = 1;
            }
        }
        if (__builtin_expect(n == 0, 0)) {
            // Canonical codes, left-aligned, grow with their length, so the
            // length is kLutBits + 1 + the number of longer-length limits the next 32 bits reach.
            const uint32_t v = __brev(w);  // first stream bit on top
            uint32_t len = kLutBits + 1;
#pragma unroll
            for (int l = kLutBits + 1; l <= 32; l++) len += ((uint64_t)v >= T.limit[l]) ? 1u : 0u;
            if (len <= 32) {
                const uint32_t off = (v >> (32 - len)) - (uint32_t)T.first_code[len];
                if (off >= T.cnt_len[len]) ok = false;
                sym0 = T.sorted_sym[(T.first_rank[len] + off) & 255u];
                len0 = len;
                n = 1;
            } else {
                // longer than 32 bits (needs a histogram as skewed as the Fibonacci numbers): bit by bit
                uint32_t bp = widx * 32 + sh;
                uint64_t code = 0;
                uint32_t sym = 0, l = 1;
                bool found = false;
                for (; l <= (uint32_t)kMaxLen; l++) {
                    code = (code << 1) | ((fetch(bp >> 5) >> (bp & 31)) & 1u);
                    bp++;
                    const uint64_t f = T.first_code[l];
                    const uint32_t c = T.cnt_len[l];
                    if (c && code >= f && code - f < c) {
                        sym = T.sorted_sym[T.first_rank[l] + (uint32_t)(code - f)];
                        found = true;
                        break;
                    }
                }
                if (!found) ok = false;
                out.put(sym);
                i++;
                widx = bp >> 5;
                sh = bp & 31;
                lo = fetch(widx);
                hi = fetch(widx + 1);
                nxt = fetch(widx + 2);
                continue;
            }
        }
        // all symbols of the entry are consumed; those past the end of the run (they belong to the next run,
        // or are pad bits) are dropped, and where the cursor ends up after the run does not matter
        out.put(sym0);
        if (n >= 2 && i + 1 < cnt) out.put((e >> 8) & 255u);
        if (n >= 3 && i + 2 < cnt) out.put((e >> 16) & 255u);
        i += n;
        sh += len0;  // total length of the entry; at most 31 + 32: one word boundary at most
        const bool cross = sh >= 32;
        lo = cross ? hi : lo;
        hi = cross ? nxt : hi;
        widx += cross ? 1u : 0u;
        sh &= 31u;
        nxt = fetch(widx + 2);
    }
    return ok;
}

// The same for a chunk staged in LDS whose run goes to 64 consecutive bytes `out`, which 4 pad bytes of the tile
// follow.  One turn of the loop reads the 64 stream bits around the cursor once (two words, at least 33 of them
// ahead of the cursor) and looks three table entries up in them, one after the other (up to 11 bits each, so the
// third still finds its 11 bits): up to nine symbols for one read of the stream and three of the table.  An
// entry's three symbol bytes go to the current position with byte stores (one unaligned 32-bit store instead
// stalls the LDS: its counters showed 70 % of its busy time in such stalls); the next entry overwrites what was not a
// symbol, and stores past the end of the run go to the pad bytes.  An entry of no symbols (a code longer than the table) leaves the cursor where it is, so the
// entries after it in the same turn are the same one: the wavefront looks at the last entry only, and branches (as
// a whole) when one of its lanes has met such a code inside its run.
// `pw` holds the chunk's nwords words and at least kPayOverrun words of any content behind them: a run of a corrupt
// stream may read that far (every symbol moves the cursor by at most 48 bits, and a run ends after 64 symbols and
// at most two more table entries), never further.
constexpr int kPayOverrun = 104;
__device__ __forceinline__ bool decode_run_bytes(const uint32_t* pw, uint32_t nwords, uint32_t start, uint32_t cnt,
                                                 const DecTables& T, uint8_t* out) {
    constexpr uint32_t kMask = (1u << kLutBits) - 1u;
    uint32_t bit = start < 32u * nwords ? start : 32u * nwords;  // (side information of a corrupt stream)
    bool ok = true;
    uint32_t i = 0;
    while (i < cnt) {
        const uint32_t* pp = pw + (bit >> 5);
        const uint32_t lo = pp[0], hi = pp[1];
        const unsigned long long win = ((unsigned long long)hi << 32) | lo;
        uint32_t sh = bit & 31u;
        // first entry: i < 64, the store stays inside the run's 64 + 4 bytes
        uint32_t e = T.lut[lut_slot(__builtin_amdgcn_alignbit(hi, lo, sh) & kMask)];
        out[i] = (uint8_t)e;
        out[i + 1] = (uint8_t)(e >> 8);
        out[i + 2] = (uint8_t)(e >> 16);
        i += e >> 29;
        uint32_t l = (e >> 24) & 31u;
        sh += l;
        bit += l;
#pragma unroll
        for (int step = 1; step < 3; step++) {
            e = T.lut[lut_slot((uint32_t)(win >> sh) & kMask)];
            const uint32_t io = i < 64u ? i : 64u;
            out[io] = (uint8_t)e;
            out[io + 1] = (uint8_t)(e >> 8);
            out[io + 2] = (uint8_t)(e >> 16);
            i += e >> 29;
            l = (e >> 24) & 31u;
            sh += l;
            bit += l;
        }
        if (__builtin_expect(__any((e >> 29) == 0 && i < cnt), 0)) {
            if ((e >> 29) == 0 && i < cnt) {
                // A code longer than the table starts at the cursor.  The next 32 bits, first stream bit on top:
                const uint32_t* qq = pw + (bit >> 5);
                const uint32_t v = __brev(__builtin_amdgcn_alignbit(qq[1], qq[0], bit & 31u));
                uint32_t sym = 0, len = 0;
                // the second table decides most of them
                const uint32_t e2 = T.lut2[((v - T.long_base) >> T.long_shift) & ((1u << kLut2Bits) - 1)];
                if (e2) {
                    sym = e2 & 255u;
                    len = e2 >> 8;
                } else {
                    // Canonical codes, left-aligned, grow with their length, so the length is kLutBits + 1 + the
                    // number of longer-length limits the 32 bits reach (limits of the lengths below the longest one
                    // are below 2^32; the longest needs no test).  One limit at a time: this is rare, and registers
                    // it would hold for all limits at once would be the whole loop's.
                    const uint32_t top = T.max_len < 33u ? T.max_len : 33u;
                    len = kLutBits + 1;
#pragma unroll 1
                    for (uint32_t q = kLutBits + 1; q < top; q++) {
                        if (v < T.limit32[q]) break;
                        len++;
                    }
                    if (len <= 32) {
                        const uint32_t off = (v >> (32 - len)) - (uint32_t)T.first_code[len];
                        if (off >= T.cnt_len[len]) ok = false;
                        sym = T.sorted_sym[(T.first_rank[len] + off) & 255u];
                    } else {
                        // longer than 32 bits (needs a histogram as skewed as the Fibonacci numbers): bit by bit
                        unsigned long long code = 0;
                        bool found = false;
                        uint32_t bp = bit;
#pragma unroll 1
                        for (len = 1; len <= (uint32_t)kMaxLen; len++) {
                            code = (code << 1) | ((pw[bp >> 5] >> (bp & 31)) & 1u);
                            bp++;
                            const unsigned long long f = T.first_code[len];
                            const uint32_t c = T.cnt_len[len];
                            if (c && code >= f && code - f < c) {
                                sym = T.sorted_sym[T.first_rank[len] + (uint32_t)(code - f)];
                                found = true;
                                break;
                            }
                        }
                        if (!found) {
                            ok = false;
                            len = kMaxLen;
                        }
                    }
                }
                out[i] = (uint8_t)sym;
                i++;
                bit += len;
            }
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
    int ncs;           // Cpad / 32
    const uint16_t* Bp16;  // inverse operand (T^T), f16 split, in operand order
    const float* mu;   // [Cpad]
    float* xhat;       // NULL in symbols-only mode
    uint8_t* syms_out; // non-NULL in symbols-only mode
    uint32_t* err;
    // where the side information and the payload start if the stream was made with the nominal chunk size
    size_t g_off_chunk_off, g_off_sub_bits, g_off_payload;
    uint32_t g_n_chunks, g_spc;
    const void* prebuilt;  // PrebuiltTables of a code table fixed beforehand, or NULL: build them from the stream
    // chunk decoder: bytes of the basis operand at the start of its dynamic LDS, and the words of payload the LDS
    // copy of a chunk holds (larger chunks are read in place); a multiple of 64
    uint32_t lds_basis_bytes, pay_words;
    int active_steps;      // contraction steps of 16 coefficients up to the basis' last row that is not all zero
    // 8-bit reconstruction in the chunk decoder (k_decode_chunks<..., U8 = true>): the transposed 8-bit basis in
    // the operand order of the integer matrix instruction [ncs][ceil(C / 16)][64], its column sums and the mean
    // in activation units (both padded to ncs * 32), h / 256 = s_T Delta / s_x, and the output bytes
    const unsigned long long* op8;
    const int* col_sum;
    const double* mean_d;
    double factor8;
    uint8_t* out8;
};

// Header checks.  Returns false unless the header matches the arguments and the
// buffer holds every section it announces.
struct StreamView {
    uint32_t n_chunks, spc, chunk_syms, payload_words;
    uint64_t ppc;
    const uint32_t* chunk_off;
    const uint16_t* sub_bits;
    const uint32_t* payload;
    float delta;
};
__device__ __forceinline__ bool open_stream(const DecodeParams& p, StreamView* v) {
    if (p.bytes < (size_t)(kHeaderBytes + kLenTableBytes)) return false;
    const Header hd = *reinterpret_cast<const Header*>(p.stream);
    const uint64_t ppc = hd.px_per_chunk;
    const uint64_t chunk_syms64 = ppc * (uint64_t)p.C;
    bool ok = hd.magic == kMagic && hd.version == 1 && hd.bits == p.bits && hd.C == (uint32_t)p.C &&
              hd.P == (uint64_t)p.P && hd.sub_syms == (uint32_t)kSubSyms && ppc >= 1 &&
              (chunk_syms64 <= 4096 || ppc == 1) && hd.delta > 0.f;
    if (!ok) return false;
    const uint64_t nch = ((uint64_t)p.P + ppc - 1) / ppc;
    const uint32_t spc = (uint32_t)((chunk_syms64 + kSubSyms - 1) / kSubSyms);
    if (nch != hd.n_chunks || spc != hd.subs_per_chunk) return false;
    const size_t off_co = kHeaderBytes + kLenTableBytes;
    const size_t off_sub = (off_co + 4 * ((size_t)nch + 1) + 15) & ~(size_t)15;
    const size_t off_pay = (off_sub + 2 * (size_t)nch * spc + 15) & ~(size_t)15;
    if (!(p.bytes >= off_pay && (p.bytes - off_pay) / 4 >= hd.payload_words && hd.payload_words <= 0xffffffffull))
        return false;
    v->n_chunks = (uint32_t)nch;
    v->spc = spc;
    v->chunk_syms = (uint32_t)chunk_syms64;
    v->payload_words = (uint32_t)hd.payload_words;
    v->ppc = ppc;
    v->chunk_off = reinterpret_cast<const uint32_t*>(p.stream + off_co);
    v->sub_bits = reinterpret_cast<const uint16_t*>(p.stream + off_sub);
    v->payload = reinterpret_cast<const uint32_t*>(p.stream + off_pay);
    v->delta = hd.delta;
    return true;
}

constexpr int kPayWords = 918;  // LDS copy of a chunk's payload: up to ~7 bits/symbol; larger chunks read global memory

// Wide tensors and the symbols-only mode: a tile of G chunks per workgroup is decoded into an LDS tile of symbol
// bytes, one chunk per wavefront and round; the inverse transform of the tile's pixels then runs on the f16 matrix
// cores with the arithmetic of the narrow-tensor kernel below (levels exact in f16, basis entries split in two f16
// parts, two matrix instructions per 16 coefficients), as a matrix product tiled over the workgroup: the basis
// blocks of a contraction step are brought into LDS once for all the tile's pixels (see the loop).
template <int MT, int LAYOUT, bool ALIGNED4>
__global__ __launch_bounds__(512) void k_decode_tiles(DecodeParams p) {
    __shared__ __align__(16) DecTables T;
    // 8 wavefronts.  Workgroup tile in units of 32: 4 pixel tiles x 8 channel tiles (128 pixels x 256 channels, a
    // wavefront 2 x 2 of them), or 2 x 8 (64 pixels, a wavefront 1 x 2) where 128 pixels of symbols do not fit LDS.
    constexpr int PTW = MT, CTW = 8, PPW = MT / 2;  // PPW: pixel tiles per wavefront
    // the chunks' payload words (one buffer per wavefront) while decoding, the basis blocks of three contraction
    // steps afterwards: the two uses are a workgroup barrier apart
    // (a payload buffer: the chunk's words, two zero words, and the room a corrupt stream's cursor may run into)
    constexpr int kPayStride = kPayWords + 2 + kPayOverrun;
    constexpr size_t kPayBytes = sizeof(uint32_t) * 8 * kPayStride, kRingBytes = sizeof(uint4) * 3 * CTW * 2 * 64;
    __shared__ __align__(16) uint8_t s_shared[kPayBytes > kRingBytes ? kPayBytes : kRingBytes];
    uint32_t(*pay)[kPayStride] = reinterpret_cast<uint32_t(*)[kPayStride]>(s_shared);
    uint4(*s_ring)[CTW * 2][64] = reinterpret_cast<uint4(*)[CTW * 2][64]>(s_shared);
    extern __shared__ __align__(16) uint8_t symtile[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wavefront-uniform by construction
    const int half = lane >> 5, l32 = lane & 31;
    const int C = p.C;

    StreamView sv;
    if (!open_stream(p, &sv)) {
        if (tid == 0) atomicOr(p.err, FMTC_ERR_HEADER);
        return;
    }
    const int my_len = tid < 256 ? (int)p.stream[kHeaderBytes + tid] : 0;
    if (!(p.prebuilt ? load_decode_tables<512>(T, my_len, static_cast<const PrebuiltTables*>(p.prebuilt))
                     : build_decode_tables<512>(T, my_len, p.bits))) {
        if (tid == 0) atomicOr(p.err, FMTC_ERR_TABLE);
        return;
    }
    const uint32_t n_chunks = sv.n_chunks, spc = sv.spc, chunk_syms = sv.chunk_syms;
    const uint32_t payload_words = sv.payload_words;
    const uint64_t ppc = sv.ppc;
    const uint32_t* chunk_off = sv.chunk_off;
    const uint16_t* sub_bits = sv.sub_bits;
    const uint32_t* payload = sv.payload;
    const uint64_t V = (uint64_t)p.P * (uint64_t)C;
    __syncthreads();

    const float delta = sv.delta;
    const int G = p.G;
    const uint32_t n_tiles = (n_chunks + G - 1) / G;
    // 0x6400 | s is the f16 number 1024 + s: the level s - 2^(b-1) is that minus (1024 + 2^(b-1)), exactly
    const _Float16 level_off = (_Float16)(float)(1024 + (1 << (p.bits - 1)));
    const halfx2 level_off2 = {level_off, level_off};
    const int NJ = p.ncs * 2;  // steps of 16 coefficients
    // ... of which the first NJA meet basis rows that are not all zero (fewer than NJ for a truncated basis)
    const int NJA = p.active_steps < 1 ? 1 : (p.active_steps > NJ ? NJ : p.active_steps);

    // x_hat = Delta (sum q T_hi + 2^-11 sum q T_lo) + mu for one 32 x 32 tile (channel tile ct, pixel tile pt of a
    // workgroup tile of TP pixels starting at pixel px_tile0).  Accumulator r of lane l is element
    // (8*(r/4) + 4*(l/32) + r%4, l%32) of the tile: rows = pixels for NHWC, channels for NCHW.  Whole tiles are
    // stored without per-element predicates (one straight run of stores).
    auto store_tile = [&](int ct, int pt, int TP, int64_t px_tile0, floatx16& acc, const floatx16& acl) {
#pragma unroll
        for (int r = 0; r < 16; r++) acc[r] = __builtin_fmaf(acl[r], 1.f / 2048.f, acc[r]) * delta;
        if constexpr (LAYOUT == FMTC_NHWC) {
            const int c = ct * 32 + l32;
            if (c < C) {
                const float m_c = p.mu[c];
                const int px_first = pt * 32;
                float* dst = p.xhat + (px_tile0 + px_first + 4 * half) * C + c;
                if (px_first + 32 <= TP) {
#pragma unroll
                    for (int r = 0; r < 16; r++) dst[(size_t)(8 * (r >> 2) + (r & 3)) * C] = acc[r] + m_c;
                } else {
#pragma unroll
                    for (int r = 0; r < 16; r++) {
                        int pxl = px_first + 8 * (r >> 2) + 4 * half + (r & 3);
                        if (pxl < TP) dst[(size_t)(8 * (r >> 2) + (r & 3)) * C] = acc[r] + m_c;
                    }
                }
            }
        } else {
            float m_r[16];
            const int cb = ct * 32 + 4 * half;
#pragma unroll
            for (int r = 0; r < 16; r++) m_r[r] = p.mu[cb + 8 * (r >> 2) + (r & 3)];  // mu is padded to a multiple of 32
            const int pxl = pt * 32 + l32;
            if (pxl < TP) {
                const int64_t px = px_tile0 + pxl;
                const int64_t n = px / p.HW, hw = px - n * p.HW;
                float* dst = p.xhat + (n * (int64_t)C + cb) * p.HW + hw;
                if (ct * 32 + 32 <= C) {
#pragma unroll
                    for (int r = 0; r < 16; r++) dst[(int64_t)(8 * (r >> 2) + (r & 3)) * p.HW] = acc[r] + m_r[r];
                } else {
#pragma unroll
                    for (int r = 0; r < 16; r++) {
                        int c = cb + 8 * (r >> 2) + (r & 3);
                        if (c < C) dst[(int64_t)(8 * (r >> 2) + (r & 3)) * p.HW] = acc[r] + m_r[r];
                    }
                }
            }
        }
    };

    for (uint32_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        // ---- variable length decoding into the LDS tile ----
        for (int j = wave; j < G; j += 8) {
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
            const uint32_t start = wave_exclusive_scan(run_bits, lane);
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
                if (cnt) {
                    // Chunk sizes that are a multiple of 64 (every run starts a 68-byte slot of the tile, and only the
                    // tensor's last run can be short) take the decoder of the narrow kernel: three table entries per
                    // read of the stream.  It stores up to three bytes past a run's last symbol: with other chunk sizes
                    // those would be the first symbols of the next chunk, which another wavefront writes.
                    if ((chunk_syms & 63u) == 0) ok_run = decode_run_bytes(pw, nwords, start, cnt, T, symtile + sym_addr(nbase));
                    else ok_run = decode_run<true>(pw, nullptr, nwords, start, cnt, T, ByteOut(symtile, nbase));
                }
                // the next chunk of this wavefront overwrites pay[]: all lanes are done reading here
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                __builtin_amdgcn_wave_barrier();
            } else if (cnt) {
                // a chunk too large for the LDS copy is read in place
                ok_run = decode_run<false>(nullptr, payload + w0, nwords, start, cnt, T, ByteOut(symtile, nbase));
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
                for (uint32_t n = 4 * tid; n < tile_syms; n += 2048)
                    *reinterpret_cast<uint32_t*>(p.syms_out + tile_s0 + n) =
                        *reinterpret_cast<const uint32_t*>(symtile + sym_addr(n));
            } else {
                for (uint32_t n = tid; n < tile_syms; n += 512) p.syms_out[tile_s0 + n] = symtile[sym_addr(n)];
            }
        } else {
            // ---- inverse quantizer + inverse transform: a tiled matrix product over the workgroup's pixels ----
            // The tile of PTW x 32 pixels times CTW x 32 output channels is shared out 2 x 2 per wavefront; the
            // contraction runs over the coefficients 16 at a time.  The basis (both f16 parts of CTW tiles, 16 bytes
            // per lane and block, operand order) goes from L2 straight into a ring of three LDS slots two steps
            // ahead -- once per workgroup and step, for all its pixels; the loads are counted by hand (see
            // load_to_lds).  The other operand is read from the symbol tile: lane (pixel, h) takes the eight symbols
            // 16 ks + 8 h .. + 7 of its pixel and turns them into f16 levels with two byte permutes each.
            const int64_t px_tile0 = (int64_t)first_ch * (int64_t)ppc;
            int TP = (int)(tile_syms / (uint32_t)C);  // pixels in this tile
            if (TP > PTW * 32) TP = PTW * 32;         // (a stream with other chunk geometry than the grid assumed)
            const int n_cg = (p.ncs + CTW - 1) / CTW;
            const int ctp = wave & 3;   // this wavefront's pair of channel tiles ...
            const int ptp = wave >> 2;  // ... and its PPW pixel tiles
            constexpr int BPW = CTW * 2 / 8;  // basis blocks a wavefront brings per step
            for (int cg = blockIdx.y; cg < n_cg; cg += gridDim.y) {
                const int ct_base = cg * CTW;
                floatx16 acc[2][PPW], acl[2][PPW];
#pragma unroll
                for (int a = 0; a < 2; a++)
#pragma unroll
                    for (int b = 0; b < PPW; b++)
#pragma unroll
                        for (int r = 0; r < 16; r++) { acc[a][b][r] = 0.f; acl[a][b][r] = 0.f; }
                uint32_t rowbase[PPW];
#pragma unroll
                for (int b = 0; b < PPW; b++) {
                    int pxl = (PPW * ptp + b) * 32 + l32;
                    if (pxl > TP - 1) pxl = TP - 1;  // rows past the tile repeat the last pixel; never stored
                    if (pxl < 0) pxl = 0;
                    rowbase[b] = (uint32_t)pxl * (uint32_t)C + 8u * half;
                }
                // steps past the end repeat the last one: the number of loads in flight is the same in every step
                auto issue = [&](int ks) {
                    const int slot = ks % 3;
                    ks = ks < NJA ? ks : NJA - 1;
#pragma unroll
                    for (int q = 0; q < BPW; q++) {
                        const int blk = wave * BPW + q;  // (channel tile blk / 2, part blk % 2)
                        int ct = ct_base + (blk >> 1);
                        ct = ct < p.ncs ? ct : p.ncs - 1;  // tiles past the end repeat the last; never stored
                        load_to_lds<16>(reinterpret_cast<const uint4*>(p.Bp16) + (((size_t)ct * NJ + ks) * 2 + (blk & 1)) * 64 + lane,
                                        &s_ring[slot][blk][0]);
                    }
                };
                issue(0);
                issue(1);
                for (int ks = 0; ks < NJA; ks++) {
                    wait_loads<BPW>();  // this wavefront's blocks of step ks have landed
                    __syncthreads();    // everybody's have, and everybody is done with the slot of step ks - 1
                    issue(ks + 2);
                    halfx8 bh[2], bl[2], q[PPW];
#pragma unroll
                    for (int a = 0; a < 2; a++) {
                        bh[a] = __builtin_bit_cast(halfx8, s_ring[ks % 3][(2 * ctp + a) * 2][lane]);
                        bl[a] = __builtin_bit_cast(halfx8, s_ring[ks % 3][(2 * ctp + a) * 2 + 1][lane]);
                    }
#pragma unroll
                    for (int b = 0; b < PPW; b++) {
                        // (coefficients past C meet zero basis entries; whatever level the tile's bytes give there
                        // does not count)
                        const uint32_t n = rowbase[b] + 16u * (uint32_t)ks;
                        uint32_t w0, w1;
                        if constexpr (ALIGNED4) {
                            w0 = *reinterpret_cast<const uint32_t*>(symtile + sym_addr(n));
                            w1 = *reinterpret_cast<const uint32_t*>(symtile + sym_addr(n + 4));
                        } else {
                            w0 = (uint32_t)symtile[sym_addr(n)] | ((uint32_t)symtile[sym_addr(n + 1)] << 8) |
                                 ((uint32_t)symtile[sym_addr(n + 2)] << 16) | ((uint32_t)symtile[sym_addr(n + 3)] << 24);
                            w1 = (uint32_t)symtile[sym_addr(n + 4)] | ((uint32_t)symtile[sym_addr(n + 5)] << 8) |
                                 ((uint32_t)symtile[sym_addr(n + 6)] << 16) | ((uint32_t)symtile[sym_addr(n + 7)] << 24);
                        }
                        const halfx2 q01 = __builtin_bit_cast(halfx2, __builtin_amdgcn_perm(0x64646464u, w0, 0x05010400u)) - level_off2;
                        const halfx2 q23 = __builtin_bit_cast(halfx2, __builtin_amdgcn_perm(0x64646464u, w0, 0x07030602u)) - level_off2;
                        const halfx2 q45 = __builtin_bit_cast(halfx2, __builtin_amdgcn_perm(0x64646464u, w1, 0x05010400u)) - level_off2;
                        const halfx2 q67 = __builtin_bit_cast(halfx2, __builtin_amdgcn_perm(0x64646464u, w1, 0x07030602u)) - level_off2;
                        q[b] = halfx8{q01[0], q01[1], q23[0], q23[1], q45[0], q45[1], q67[0], q67[1]};
                    }
#pragma unroll
                    for (int a = 0; a < 2; a++)
#pragma unroll
                        for (int b = 0; b < PPW; b++) {
                            if constexpr (LAYOUT == FMTC_NHWC) {
                                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(q[b], bh[a], acc[a][b], 0, 0, 0);
                                acl[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(q[b], bl[a], acl[a][b], 0, 0, 0);
                            } else {
                                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(bh[a], q[b], acc[a][b], 0, 0, 0);
                                acl[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(bl[a], q[b], acl[a][b], 0, 0, 0);
                            }
                        }
                }
                wait_loads<0>();  // the repeated loads of the last steps
                __syncthreads();  // nobody reads the ring any more: the next channel group may refill it

#pragma unroll
                for (int a = 0; a < 2; a++) {
                    const int ct = ct_base + 2 * ctp + a;
                    if (ct >= p.ncs) continue;  // wavefront-uniform
#pragma unroll
                    for (int b = 0; b < PPW; b++) {
                        const int pt = PPW * ptp + b;
                        if (pt * 32 >= TP) continue;  // wavefront-uniform
                        store_tile(ct, pt, TP, px_tile0, acc[a][b], acl[a][b]);
                    }
                }
            }
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------
// Narrow tensors (at most 160 channels after padding to 32): a chunk holds at least 25
// pixels, so the wavefront that decoded it has whole matrix tiles of its own.  The inverse
// transform runs on the f16 matrix cores (v_mfma_f32_32x32x16_f16): the levels s - 2^(b-1)
// are small integers, exact in f16, and every basis entry is split in two f16 parts,
// T = hi + lo / 2^11 (22 significant bits; see pack_operand16 on the host), so
//   x_hat = Delta (sum q T_hi + 2^-11 sum q T_lo) + mu
// with exact products and fp32 accumulation: two instructions per 16 coefficients where the
// fp32 instruction needs eight four times as long.  The basis is copied once per workgroup
// into LDS in operand order; lane (row, half) of the other operand reads the eight symbols
// 16j + 8*half + e of its pixel (the contraction index may be walked in any order as long as
// both operands agree on it).  Delta and mu are applied in the epilogue.
// ---------------------------------------------------------------------------
typedef int intx16 __attribute__((ext_vector_type(16)));
constexpr int kChunkTileBytes = 4096 + 4096 / 16 + 64;  // symbols, 4 pad bytes per run, slack for padded reads

// WAVES wavefronts per workgroup (4 or 8): one per SIMD where the chunks do not outnumber the SIMDs, two where
// they do (the second hides the latencies of the first; the workgroup still holds one copy of the basis).
// U8: the tile's symbols go through the 8-bit basis on the integer matrix cores instead (v_mfma_i32_32x32x16_i8;
// exact sums, one fused fp64 multiply-add and one rounding per value, 8-bit activations out); the 8-bit basis
// takes the f16 basis' place in LDS.
// CFIX: the tensor's channel count if the kernel is built for one (the launcher checks it; 0: any), which makes every
// row stride a constant.
// LOG: only the upper f16 parts of the basis are kept in LDS; the lower parts, whose products are the small
// correction, are read from global memory (the cache serves them: every wavefront of the device reads the same few
// tens of KB) while the matrix instructions of the upper parts run.  Half the LDS per workgroup buys a third
// wavefront per SIMD for 128 to 160 channels.
template <int NCT, int LAYOUT, bool ALIGNED4, int WAVES, bool U8 = false, int CFIX = 0, bool LOG = false, int NLO = 0>
__global__ __launch_bounds__(WAVES * 64) __attribute__((amdgpu_waves_per_eu(WAVES / 4, WAVES / 4))) void k_decode_chunks(DecodeParams p) {
    constexpr int THREADS = WAVES * 64;
    __shared__ __align__(16) DecTables T;
    __shared__ __align__(16) uint8_t symtile[WAVES][kChunkTileBytes];
    __shared__ float s_mu[NCT * 32];
    // 8-bit variant: column sums and means of the channels (read for every value of the epilogue)
    __shared__ int s_col_sum[U8 ? NCT * 32 : 1];
    __shared__ double s_mean_d[U8 ? NCT * 32 : 1];
    // the basis operand [NCT][NJ][2][64], then per wavefront the chunk's payload words and room for a corrupt
    // stream's overrun
    extern __shared__ __align__(16) uint4 basis16[];
    constexpr int NJ = NCT * 2;  // steps of 16 coefficients
    const uint32_t pay_cap = p.pay_words;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wavefront-uniform by construction
    const int half = lane >> 5, l32 = lane & 31;
    const int C = CFIX ? CFIX : p.C;
    static_assert(!(LOG && U8), "the 8-bit basis has one part");
    // The variants for many chunks (tens of MB of output and more) store the activations with the streaming hint:
    // written through the 256 MB memory-side cache, a large tensor leaves its write-back to whatever kernel runs
    // next.  (Measured on the 205 MB tensor: the decoder, which has memory bandwidth to spare, takes 7 us longer, and
    // the projection after it, which no longer shares the memory with that write-back, 14 us less.)
    constexpr bool kStreamOut = !U8 && (WAVES >= 12 || LOG);

    // loads that do not depend on the header go out first: the code length table and the basis
    int my_len = 0;
    if (tid < 256 && p.bytes >= (size_t)(kHeaderBytes + kLenTableBytes)) my_len = p.stream[kHeaderBytes + tid];
    // the basis goes from global memory straight into LDS (no registers in between), 16 bytes per lane and
    // instruction: lane l of a wavefront lands at the wavefront's LDS base + 16 l
    constexpr int kBasisPieces = NCT * NJ * 2 * 64;  // 16-byte pieces of the basis, a multiple of 64
    if constexpr (U8) {
        // the 8-bit basis operand, [NCT][NS][64] entries of 8 bytes, goes into the same dynamic LDS
        const int n16 = NCT * ((C + 15) / 16) * 32;  // 16-byte pieces
        const uint4* src = reinterpret_cast<const uint4*>(p.op8);
        for (int i = tid; i < n16; i += THREADS) basis16[i] = src[i];
    }
    if constexpr (!U8 && !LOG) {
        const uint4* src = reinterpret_cast<const uint4*>(p.Bp16);
#pragma unroll
        for (int i = 0; i < (kBasisPieces + THREADS - 1) / THREADS; i++)
            if (THREADS * i + 64 * wave < kBasisPieces)  // whole wavefronts
                __builtin_amdgcn_global_load_lds(src + tid + THREADS * i, &basis16[THREADS * i + 64 * wave], 16, 0, 0);
    }
    if constexpr (LOG) {
        // block g = (channel tile, step) of the upper parts: 64 pieces at [g][0][64] of the operand, to [g][64] in LDS
        const uint4* src = reinterpret_cast<const uint4*>(p.Bp16);
        for (int g = wave; g < NCT * NJ; g += WAVES)
            __builtin_amdgcn_global_load_lds(src + (size_t)g * 128 + lane, &basis16[g * 64], 16, 0, 0);
        // ... and the lower parts of the first NLO channel tiles behind them
        for (int g = wave; g < NLO * NJ; g += WAVES)
            __builtin_amdgcn_global_load_lds(src + (size_t)g * 128 + 64 + lane, &basis16[(NCT * NJ + g) * 64], 16, 0, 0);
    }
    // The first chunk's offsets, run sizes and payload are requested before the header has arrived, at the places
    // the nominal chunk size puts them: three dependent memory round trips (header, offsets, payload) become
    // two that overlap with the table build.  The guess is checked against the header below; a stream made with
    // another chunk size loads them again.  Nothing outside [stream, stream + bytes) is touched either way.
    // (chunk c goes to workgroup c mod gridDim.x: a last, partly filled round of chunks is spread over all compute
    // units, one wavefront each, instead of filling a few of them)
    const uint32_t ch_first = (uint32_t)wave * gridDim.x + blockIdx.x;
    // this wavefront's LDS copy of a chunk's payload: pay_cap words and the overrun room
    uint32_t* pw = reinterpret_cast<uint32_t*>(reinterpret_cast<uint8_t*>(basis16) + p.lds_basis_bytes) +
                   (size_t)wave * (pay_cap + (uint32_t)kPayOverrun);
    // Words [w0, w0 + n) of the payload go from global memory straight into that copy, 4 bytes per lane and
    // instruction, no registers in between; lanes past the chunk's end load nothing (what lies behind the chunk in
    // LDS is whatever was there: the decoder never takes a symbol of its run from it).  Asynchronous: wait_loads<0>()
    // before the copy is read.
    auto request_payload = [&](const uint32_t* payload, uint32_t w0, uint32_t n) {
        const uint32_t* src = payload + w0;
        for (uint32_t k = 0; 64u * k < n; k++) {  // wavefront-uniform trip count
            const uint32_t i = (uint32_t)lane + 64u * k;
            if (i < n) load_to_lds<4>(src + i, pw + 64u * k);
        }
    };
    const bool guess = p.g_off_payload <= p.bytes && ch_first < p.g_n_chunks;
    uint32_t pre_w0 = 0, pre_w1 = 0, pre_run = 0;
    bool pay_pre = false;
    if (guess) {
        const uint32_t* co = reinterpret_cast<const uint32_t*>(p.stream + p.g_off_chunk_off);
        const uint16_t* sb = reinterpret_cast<const uint16_t*>(p.stream + p.g_off_sub_bits);
        pre_w0 = co[ch_first];
        pre_w1 = co[ch_first + 1];
        pre_run = ((uint32_t)lane < p.g_spc) ? sb[(size_t)ch_first * p.g_spc + lane] : 0u;
        const size_t cap_words = (p.bytes - p.g_off_payload) / 4;
        const uint32_t gw0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)pre_w0);
        const uint32_t gw1 = (uint32_t)__builtin_amdgcn_readfirstlane((int)pre_w1);
        pay_pre = gw0 <= gw1 && (size_t)gw1 <= cap_words && gw1 - gw0 <= pay_cap;
        if (pay_pre) request_payload(reinterpret_cast<const uint32_t*>(p.stream + p.g_off_payload), gw0, gw1 - gw0);
    }
    StreamView sv;
    if (!open_stream(p, &sv)) {
        if (tid == 0 && blockIdx.x == 0) atomicOr(p.err, FMTC_ERR_HEADER);
        return;
    }
    const bool guess_valid = guess && sv.n_chunks == p.g_n_chunks && sv.spc == p.g_spc;  // same section offsets
    const uint32_t guess_w0 = pre_w0, guess_w1 = pre_w1;
    if (!guess_valid) {
        pre_w0 = 0; pre_w1 = 0; pre_run = 0;
        if (ch_first < sv.n_chunks) {
            pre_w0 = sv.chunk_off[ch_first];
            pre_w1 = sv.chunk_off[ch_first + 1];
            pre_run = ((uint32_t)lane < sv.spc) ? sv.sub_bits[(size_t)ch_first * sv.spc + lane] : 0u;
        }
    }
    if constexpr (!U8) {
        if (tid < NCT * 32) s_mu[tid] = p.mu[tid];
    } else {
        if (tid < NCT * 32) {  // (both arrays are padded to NCT * 32 entries)
            s_col_sum[tid] = p.col_sum[tid];
            s_mean_d[tid] = p.mean_d[tid];
        }
    }
    if (!(p.prebuilt ? load_decode_tables<THREADS>(T, my_len, static_cast<const PrebuiltTables*>(p.prebuilt))
                     : build_decode_tables<THREADS>(T, my_len, p.bits))) {
        if (tid == 0 && blockIdx.x == 0) atomicOr(p.err, FMTC_ERR_TABLE);
        return;
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wavefront's part of the basis has landed in LDS
    __syncthreads();
    const uint32_t n_chunks = sv.n_chunks, spc = sv.spc, chunk_syms = sv.chunk_syms;
    const uint32_t payload_words = sv.payload_words;
    const uint64_t V = (uint64_t)p.P * (uint64_t)C;
    const float delta = sv.delta;
    // contraction steps that meet a non-zero row of the basis (all of them unless the basis is truncated)
    const int NJA = p.active_steps < 1 ? 1 : (p.active_steps > NJ ? NJ : p.active_steps);
    // 0x6400 | s is the f16 number 1024 + s: the level s - 2^(b-1) is that minus (1024 + 2^(b-1)), exactly
    const _Float16 level_off = (_Float16)(float)(1024 + (1 << (p.bits - 1)));
    const halfx2 level_off2 = {level_off, level_off};
    uint8_t* tile = symtile[wave];

    // Side information and payload of a chunk are requested one chunk ahead: its payload words right after the
    // variable length decoding of the chunk before it (the LDS copy is free then; they arrive during the inverse
    // transform), offsets and run sizes of the chunk after it once those words have landed (they arrive during the
    // variable length decoding) -- a chunk would otherwise start with two dependent memory round trips.  cur_*:
    // what is at hand for the chunk of this turn; pay_*: the offsets the words in the LDS copy were requested for.
    uint32_t cur_w0 = pre_w0, cur_w1 = pre_w1, cur_run = pre_run;
    bool pay_ok = guess_valid && pay_pre;
    uint32_t pay_w0 = guess_w0, pay_w1 = guess_w1;
    const uint32_t ch_step = gridDim.x * WAVES;
    for (uint32_t ch = ch_first; ch < n_chunks; ch += ch_step) {
        // ---- variable length decoding of the chunk into the wavefront's tile ----
        const uint64_t c0 = (uint64_t)ch * chunk_syms;
        const uint32_t clen = (uint32_t)((V - c0 < chunk_syms) ? (V - c0) : chunk_syms);
        uint32_t w0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)cur_w0);
        uint32_t w1 = (uint32_t)__builtin_amdgcn_readfirstlane((int)cur_w1);
        if (w0 > w1 || w1 > payload_words) {
            if (lane == 0) atomicOr(p.err, FMTC_ERR_OFFSETS);
            w0 = 0; w1 = 0;
        }
        const uint32_t run_bits = cur_run;
        const uint32_t nwords = w1 - w0;
        const bool staged = nwords <= pay_cap;
        // (whatever was requested for the LDS copy has landed before it is read or requested again; this also waits
        // for the stores of the chunk before)
        wait_loads<0>();
        if (staged && !(pay_ok && w0 == pay_w0 && w1 == pay_w1)) {
            request_payload(sv.payload, w0, nwords);
            wait_loads<0>();
        }
        const uint32_t nch = ch + ch_step;
        const bool have_next = nch < n_chunks && nch > ch;  // wavefront-uniform
        if (have_next) {
            cur_w0 = sv.chunk_off[nch];
            cur_w1 = sv.chunk_off[nch + 1];
            cur_run = ((uint32_t)lane < spc) ? sv.sub_bits[(size_t)nch * spc + lane] : 0u;
        }
        const uint32_t start = wave_exclusive_scan(run_bits, lane);
        const uint32_t r0 = (uint32_t)lane * kSubSyms;
        const uint32_t cnt = (r0 < clen) ? ((clen - r0 < (uint32_t)kSubSyms) ? clen - r0 : (uint32_t)kSubSyms) : 0u;
        bool ok_run = true;
        if (staged) {
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            // run `lane` goes to bytes [68 * lane, 68 * lane + 64) of the tile (sym_addr), 4 pad bytes behind it
            if (cnt) ok_run = decode_run_bytes(pw, nwords, start, cnt, T, tile + 68u * (uint32_t)lane);
        } else if (cnt) {
            ok_run = decode_run<false>(nullptr, sv.payload + w0, nwords, start, cnt, T, ByteOut(tile, r0));
        }
        // the next chunk's payload words: in flight during this chunk's inverse transform (every lane is done with
        // the LDS copy: the reads of a wavefront complete in order, and each lane has used its last one)
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        pay_ok = false;
        if (have_next) {
            pay_w0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)cur_w0);
            pay_w1 = (uint32_t)__builtin_amdgcn_readfirstlane((int)cur_w1);
            pay_ok = pay_w0 <= pay_w1 && pay_w1 <= payload_words && pay_w1 - pay_w0 <= pay_cap;
            if (pay_ok) request_payload(sv.payload, pay_w0, pay_w1 - pay_w0);
        }
        if (!ok_run) atomicOr(p.err, FMTC_ERR_CODE);
        // the symbols of all lanes are in place before any lane reads them: one wavefront, LDS in order
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();

        // ---- inverse quantizer + inverse transform of the chunk's pixels ----
        const int TP = (int)(clen / (uint32_t)C);
        const int64_t px_chunk0 = (int64_t)ch * (int64_t)sv.ppc;
        for (int pt = 0; pt * 32 < TP; pt++) {
            int pxl = pt * 32 + l32;
            if (pxl > TP - 1) pxl = TP - 1;  // rows past the chunk repeat its last pixel; never stored
            const uint32_t rowbase = (uint32_t)pxl * (uint32_t)C + 8u * (uint32_t)half;
            if constexpr (U8) {
                // Operands: lane (l32, half) holds the 8 symbols 16j + 8*half .. + 7 of its pixel as (s - 128),
                // and of the basis the same 8 coefficients of channel row perm(l32) of tile ct (rows permuted so
                // that a lane ends up with channels ct*32 + 16*half .. + 15 of its pixel).  Symbols past C meet
                // zero basis bytes.
                const int NS = (C + 15) / 16;  // <= NJ
                const unsigned long long* op8_lds = reinterpret_cast<const unsigned long long*>(basis16);
                const int hk = 1 << (p.bits - 1);
                long b[NJ];
#pragma unroll
                for (int j = 0; j < NJ; j++) {
                    const uint32_t n = rowbase + 16u * (uint32_t)j;
                    uint32_t w0 = 0, w1 = 0;
                    if (j < NS) {
                        if constexpr (ALIGNED4) {
                            w0 = *reinterpret_cast<const uint32_t*>(tile + sym_addr(n));
                            w1 = *reinterpret_cast<const uint32_t*>(tile + sym_addr(n + 4));
                        } else {
                            w0 = (uint32_t)tile[sym_addr(n)] | ((uint32_t)tile[sym_addr(n + 1)] << 8) |
                                 ((uint32_t)tile[sym_addr(n + 2)] << 16) | ((uint32_t)tile[sym_addr(n + 3)] << 24);
                            w1 = (uint32_t)tile[sym_addr(n + 4)] | ((uint32_t)tile[sym_addr(n + 5)] << 8) |
                                 ((uint32_t)tile[sym_addr(n + 6)] << 16) | ((uint32_t)tile[sym_addr(n + 7)] << 24);
                        }
                    }
                    b[j] = (long)((((unsigned long long)w1 << 32) | w0) ^ 0x8080808080808080ull);
                }
                const int my_px = pt * 32 + l32;
                const int64_t px = px_chunk0 + my_px;
#pragma unroll
                for (int ct = 0; ct < NCT; ct++) {
                    intx16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
                    for (int j = 0; j < NJ; j++)
                        if (j < NS)
                            acc = __builtin_amdgcn_mfma_i32_32x32x16_i8((long)op8_lds[(ct * NS + j) * 64 + lane], b[j], acc, 0, 0, 0);
                    const int r0 = ct * 32 + 16 * half;
                    uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
                    for (int v = 0; v < 16; v++) {
                        const int r = r0 + v;  // < NCT * 32: the per-channel arrays are padded to that
                        const int m = acc[v] + (128 - hk) * s_col_sum[r];
                        const double t = fmin(fmax(rint(fma((double)m, p.factor8, s_mean_d[r])), 0.0), 255.0);
                        w[v >> 2] |= (uint32_t)(int)t << (8 * (v & 3));
                    }
                    if (my_px < TP && r0 < C) {
                        if constexpr (LAYOUT == FMTC_NHWC) {
                            uint8_t* q = p.out8 + (size_t)px * (size_t)C + (size_t)r0;
                            if ((C % 16) == 0) {
                                *reinterpret_cast<uint4*>(q) = make_uint4(w[0], w[1], w[2], w[3]);
                            } else {
#pragma unroll
                                for (int v = 0; v < 16; v++)
                                    if (r0 + v < C) q[v] = (uint8_t)(w[v >> 2] >> (8 * (v & 3)));
                            }
                        } else {
                            const int64_t n = px / p.HW, hw = px - n * p.HW;
#pragma unroll
                            for (int v = 0; v < 16; v++)
                                if (r0 + v < C)
                                    p.out8[((size_t)n * (size_t)C + (size_t)(r0 + v)) * (size_t)p.HW + (size_t)hw] =
                                        (uint8_t)(w[v >> 2] >> (8 * (v & 3)));
                        }
                    }
                }
                continue;
            }
            // the levels of this lane's pixel as f16 operands, all contraction steps (coefficients past C meet zero
            // basis entries; whatever finite level the tile's bytes give there does not count)
            halfx8 q[NJ];
#pragma unroll
            for (int j = 0; j < NJ; j++) {
                const uint32_t n = rowbase + 16u * (uint32_t)j;
                uint32_t w0, w1;
                if constexpr (ALIGNED4) {
                    w0 = *reinterpret_cast<const uint32_t*>(tile + sym_addr(n));
                    w1 = *reinterpret_cast<const uint32_t*>(tile + sym_addr(n + 4));
                } else {
                    w0 = (uint32_t)tile[sym_addr(n)] | ((uint32_t)tile[sym_addr(n + 1)] << 8) |
                         ((uint32_t)tile[sym_addr(n + 2)] << 16) | ((uint32_t)tile[sym_addr(n + 3)] << 24);
                    w1 = (uint32_t)tile[sym_addr(n + 4)] | ((uint32_t)tile[sym_addr(n + 5)] << 8) |
                         ((uint32_t)tile[sym_addr(n + 6)] << 16) | ((uint32_t)tile[sym_addr(n + 7)] << 24);
                }
                const halfx2 q01 = __builtin_bit_cast(halfx2, __builtin_amdgcn_perm(0x64646464u, w0, 0x05010400u)) - level_off2;
                const halfx2 q23 = __builtin_bit_cast(halfx2, __builtin_amdgcn_perm(0x64646464u, w0, 0x07030602u)) - level_off2;
                const halfx2 q45 = __builtin_bit_cast(halfx2, __builtin_amdgcn_perm(0x64646464u, w1, 0x05010400u)) - level_off2;
                const halfx2 q67 = __builtin_bit_cast(halfx2, __builtin_amdgcn_perm(0x64646464u, w1, 0x07030602u)) - level_off2;
                q[j] = halfx8{q01[0], q01[1], q23[0], q23[1], q45[0], q45[1], q67[0], q67[1]};
            }
            // One channel tile at a time: one pair of accumulators, the contraction, the epilogue, the stores (all
            // tiles at once would hold 2 NCT accumulators: the registers of a third wavefront per SIMD).
            // LOG: the lower parts of the first NLO channel tiles sit in LDS behind the upper parts (as many as fit
            // beside the wavefronts' buffers), those of the others come from global memory.  The tiles with everything in
            // LDS go first, and the others' lower parts are requested before them: a round trip to the cache takes 1 to
            // 1.5 us under this kernel's load, a channel tile's arithmetic a third of that.  At most two wavefronts per
            // SIMD have the registers to request all of them at the top; three request one tile's, and the next tile's
            // when that one's matrix instructions have issued.
            constexpr int NG = LOG ? NCT - NLO : 0;
            constexpr bool kLoAll = LOG && WAVES <= 8 && NG <= 2;
            uint4 lo_g[kLoAll ? (NG > 0 ? NG : 1) : 1][LOG ? NJ : 1];
            auto request_lo = [&](int ct, uint4 (&dst)[LOG ? NJ : 1]) __attribute__((always_inline)) {
                if constexpr (LOG) {
                    const uint4* lo_src = reinterpret_cast<const uint4*>(p.Bp16) + ((size_t)(ct * NJ) * 2 + 1) * 64 + lane;
#pragma unroll
                    for (int j = 0; j < NJ; j++)
                        if (j < NJA) dst[j] = lo_src[(size_t)j * 128];
                }
            };
            if constexpr (LOG && NG > 0) {
                request_lo(NLO, lo_g[0]);
                if constexpr (kLoAll) {
#pragma unroll
                    for (int g = 1; g < NG; g++) request_lo(NLO + g, lo_g[g]);
                }
            }
#pragma unroll
            for (int ct = 0; ct < NCT; ct++) {
                floatx16 acc, acl;
#pragma unroll
                for (int r = 0; r < 16; r++) { acc[r] = 0.f; acl[r] = 0.f; }
                if constexpr (LOG) {
#pragma unroll
                    for (int j = 0; j < NJ; j++) {
                        if (j >= NJA) continue;  // wavefront-uniform (truncation, and padding rows of the last tile)
                        const halfx8 bh = __builtin_bit_cast(halfx8, basis16[(ct * NJ + j) * 64 + lane]);
                        if constexpr (LAYOUT == FMTC_NHWC) acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(q[j], bh, acc, 0, 0, 0);
                        else acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(bh, q[j], acc, 0, 0, 0);
                    }
#pragma unroll
                    for (int j = 0; j < NJ; j++) {
                        if (j >= NJA) continue;
                        halfx8 bl;
                        if (ct < NLO) bl = __builtin_bit_cast(halfx8, basis16[((NCT + ct) * NJ + j) * 64 + lane]);
                        else bl = __builtin_bit_cast(halfx8, lo_g[kLoAll ? ct - NLO : 0][j]);
                        if constexpr (LAYOUT == FMTC_NHWC) acl = __builtin_amdgcn_mfma_f32_32x32x16_f16(q[j], bl, acl, 0, 0, 0);
                        else acl = __builtin_amdgcn_mfma_f32_32x32x16_f16(bl, q[j], acl, 0, 0, 0);
                    }
                    if constexpr (!kLoAll) {
                        if (ct >= NLO && ct + 1 < NCT) request_lo(ct + 1, lo_g[0]);
                    }
                } else {
#pragma unroll
                for (int j = 0; j < NJ; j++) {
                    if (j >= NJA) continue;  // wavefront-uniform: steps past the basis' last non-zero row (truncation)
                    const halfx8 bh = __builtin_bit_cast(halfx8, basis16[((ct * NJ + j) * 2) * 64 + lane]);
                    const halfx8 bl = __builtin_bit_cast(halfx8, basis16[((ct * NJ + j) * 2 + 1) * 64 + lane]);
                    if constexpr (LAYOUT == FMTC_NHWC) {
                        acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(q[j], bh, acc, 0, 0, 0);
                        acl = __builtin_amdgcn_mfma_f32_32x32x16_f16(q[j], bl, acl, 0, 0, 0);
                    } else {
                        acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(bh, q[j], acc, 0, 0, 0);
                        acl = __builtin_amdgcn_mfma_f32_32x32x16_f16(bl, q[j], acl, 0, 0, 0);
                    }
                }
                }
#pragma unroll
                for (int r = 0; r < 16; r++) acc[r] = __builtin_fmaf(acl[r], 1.f / 2048.f, acc[r]);
                // accumulator r of lane l is element (8*(r/4) + 4*(l/32) + r%4, l%32) of the 32x32 tile
                if constexpr (LAYOUT == FMTC_NHWC) {
                    const int c = ct * 32 + l32;
                    if (c < C) {
                        const float m_c = s_mu[c];
                        float* dst = p.xhat + (px_chunk0 + pt * 32 + 4 * half) * C + c;
                        if (pt * 32 + 32 <= TP && C == NCT * 32) {
                            // (the usual case, with the row stride a constant: the stores' offsets are immediates
                            // instead of sixteen 64-bit values in registers)
                            if constexpr (kStreamOut) {
#pragma unroll
                                for (int r = 0; r < 16; r++)
                                    __builtin_nontemporal_store(__builtin_fmaf(acc[r], delta, m_c),
                                                                &dst[(size_t)(8 * (r >> 2) + (r & 3)) * (NCT * 32)]);
                            } else {
#pragma unroll
                                for (int r = 0; r < 16; r++)
                                    dst[(size_t)(8 * (r >> 2) + (r & 3)) * (NCT * 32)] = __builtin_fmaf(acc[r], delta, m_c);
                            }
                        } else if (CFIX != 0 && CFIX != NCT * 32) {
                            // (a channel count known at build time that is no multiple of 32: the same, with the
                            // rows past the chunk's last pixel left out)
                            // (a whole chunk of such a tensor ends inside the last eight rows of the tile: the rows before
                            // them need no test -- wavefront-uniform -- and the stores go out in one run)
                            const bool first24 = pt * 32 + 24 <= TP;
#pragma unroll
                            for (int r = 0; r < 16; r++)
                                if ((r < 12 && first24) || pt * 32 + 8 * (r >> 2) + 4 * half + (r & 3) < TP) {
                                    float* at = &dst[(size_t)(8 * (r >> 2) + (r & 3)) * (CFIX ? CFIX : 1)];
                                    if constexpr (kStreamOut) __builtin_nontemporal_store(__builtin_fmaf(acc[r], delta, m_c), at);
                                    else *at = __builtin_fmaf(acc[r], delta, m_c);
                                }
                        } else if (pt * 32 + 32 <= TP) {
#pragma unroll
                            for (int r = 0; r < 16; r++)
                                dst[(size_t)(8 * (r >> 2) + (r & 3)) * C] = __builtin_fmaf(acc[r], delta, m_c);
                        } else {
#pragma unroll
                            for (int r = 0; r < 16; r++)
                                if (pt * 32 + 8 * (r >> 2) + 4 * half + (r & 3) < TP)
                                    dst[(size_t)(8 * (r >> 2) + (r & 3)) * C] = __builtin_fmaf(acc[r], delta, m_c);
                        }
                    }
                } else {
                    const int my_px = pt * 32 + l32;
                    if (my_px < TP) {
                        const int64_t px = px_chunk0 + my_px;
                        const int64_t n = px / p.HW, hw = px - n * p.HW;
                        const int cb = ct * 32 + 4 * half;
                        float* dst = p.xhat + (n * (int64_t)C + cb) * p.HW + hw;
#pragma unroll
                        for (int r = 0; r < 16; r++) {
                            const int co = 8 * (r >> 2) + (r & 3);
                            if (cb + co < C) dst[(int64_t)co * p.HW] = __builtin_fmaf(acc[r], delta, s_mu[cb + co]);
                        }
                    }
                }
            }
        }
        // the next chunk of this wavefront overwrites the tile and pay[]: all lanes are done reading here
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}

hipError_t launch_decode(const BasisDevice* b, const uint8_t* d_stream, size_t bytes, const Geometry& g, int bits,
                         int64_t HW, int layout, float* d_xhat, uint8_t* d_syms, uint32_t* d_err, const void* d_prebuilt,
                         hipStream_t s) {
    const int C = g.C;
    const int ncs = (C + 31) / 32;
    DecodeParams p{};
    p.stream = d_stream;
    p.bytes = bytes;
    p.P = g.P;
    p.HW = HW;
    p.C = C;
    p.bits = bits;
    p.ncs = ncs;
    p.Bp16 = b ? b->inv16 : nullptr;
    p.active_steps = b ? (b->active_rows + 15) / 16 : 0;
    p.mu = b ? b->mu : nullptr;
    p.xhat = d_xhat;
    p.syms_out = d_syms;
    p.err = d_err;
    p.prebuilt = d_prebuilt;
    p.G = 1;
    p.g_off_chunk_off = g.off_chunk_off;
    p.g_off_sub_bits = g.off_sub_bits;
    p.g_off_payload = g.off_payload;
    p.g_n_chunks = g.n_chunks;
    p.g_spc = g.subs_per_chunk;
    const bool al = (C % 4) == 0;
    hipError_t el = hipSuccess;
    // (five channel tiles: channels-last only, the planar stores take more registers than are left)
    if (!d_syms && (ncs <= 4 || (ncs == 5 && layout == FMTC_NHWC))) {
        // ---- one wavefront per chunk ----
        const size_t lds_basis = sizeof(float) * (size_t)ncs * 32 * ncs * 32;
        // The LDS copy of a chunk's payload holds what a chunk takes at the fixed-length rate of `bits` per symbol
        // (which the code of the whole tensor never exceeds on average) and a little more; a chunk beyond that is
        // read in place.
        p.lds_basis_bytes = (uint32_t)lds_basis;
        p.pay_words = 128u * (uint32_t)bits + 64u;
        auto lds_dyn = [&](int wv) { return lds_basis + (size_t)wv * (p.pay_words + kPayOverrun) * 4; };
        auto lds_all = [&](int wv) { return lds_dyn(wv) + sizeof(DecTables) + (size_t)wv * kChunkTileBytes + (size_t)ncs * 128 + 64; };
        // One, two or four wavefronts per SIMD as the chunks outnumber the SIMDs of the device: the variable length
        // decoding is a chain of dependent LDS reads, and the other wavefronts' work fills its waits.  (Three channel
        // tiles need more registers, five more LDS, than two wavefronts per SIMD leave; four per SIMD fit up to two
        // channel tiles.)
        int waves = 4;
        if (g.n_chunks > 1024 && ncs != 3 && ncs != 5) waves = 8;
        if (g.n_chunks > 3072 && ncs <= 2 && C == ncs * 32 && layout == FMTC_NHWC && lds_all(16) <= 160 * 1024) waves = 16;
        // 128 to 160 channels: three wavefronts per SIMD with the lower parts of the basis left in global memory
        // (k_decode_chunks<..., LOG>); built for the channel counts 128 and 144, channels last (with a channel count
        // left open the kernel does not fit the registers of three wavefronts)
        // (144 channels: two wavefronts per SIMD, the registers of a third do not fit)
        // (the lower parts of the first `nlo` channel tiles go to LDS all the same if the bit depth's payload buffers
        // leave the room: 2 of 4 tiles at 128 channels, 3 of 5 at 144)
        const int log_waves = C == 128 ? 12 : 8;
        const int nlo_want = C == 128 ? 2 : 3;
        const size_t lo_tile = lds_basis / 2 / (size_t)ncs;  // bytes of one channel tile's lower parts
        auto lds_basis_for = [&](int nlo) { return lds_basis / 2 + (size_t)nlo * lo_tile; };
        const bool fits_lo = lds_all(log_waves) - lds_basis + lds_basis_for(nlo_want) <= 160 * 1024;
        const int nlo = fits_lo ? nlo_want : 0;
        const size_t lds_basis_log = lds_basis_for(nlo);
        const bool log12 = (C == 128 || C == 144) && layout == FMTC_NHWC && g.n_chunks > 2048 &&
                           lds_all(log_waves) - lds_basis + lds_basis_log <= 160 * 1024;
        if (log12) {
            waves = log_waves;
            p.lds_basis_bytes = (uint32_t)lds_basis_log;
        }
        const size_t lds = log12 ? lds_dyn(waves) - lds_basis + lds_basis_log : lds_dyn(waves);
        const unsigned per_cu = log12 ? 1u : (unsigned)((160 * 1024) / lds_all(waves));
        unsigned gx = (g.n_chunks + waves - 1) / waves;
        const unsigned most = waves >= 8 ? 1u : 2u;
        const unsigned cap = 256u * (per_cu < 1 ? 1u : (per_cu > most ? most : per_cu));
        if (gx > cap) gx = cap;
#define FMTC_DECC_L(NCT, LAY, AL, WV, CF, LG, NL)                                                                \
    do {                                                                                                         \
        if (lds > 16 * 1024) {                                                                                   \
            hipError_t ea = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_decode_chunks<NCT, LAY, AL, WV, false, CF, LG, NL>), \
                                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);          \
            if (ea != hipSuccess) return ea;                                                                     \
        }                                                                                                        \
        el = launch(K_DECODE, k_decode_chunks<NCT, LAY, AL, WV, false, CF, LG, NL>, dim3(gx), dim3(WV * 64), lds, s, p); \
    } while (0)
#define FMTC_DECC_F(NCT, LAY, AL, WV, CF, LG) FMTC_DECC_L(NCT, LAY, AL, WV, CF, LG, 0)
#define FMTC_DECC(NCT, LAY, AL, WV) FMTC_DECC_F(NCT, LAY, AL, WV, 0, false)
#define FMTC_DECC_N(LAY, AL)                                                                                     \
    do {                                                                                                         \
        if (ncs == 1) { if (waves == 8) FMTC_DECC(1, LAY, AL, 8); else FMTC_DECC(1, LAY, AL, 4); }               \
        else if (ncs == 2) { if (waves == 8) FMTC_DECC(2, LAY, AL, 8); else FMTC_DECC(2, LAY, AL, 4); }          \
        else if (ncs == 3) FMTC_DECC(3, LAY, AL, 4);                                                             \
        else { if (waves == 8) FMTC_DECC(4, LAY, AL, 8); else FMTC_DECC(4, LAY, AL, 4); }                        \
    } while (0)
        if (waves == 16) { if (ncs == 1) FMTC_DECC_F(1, FMTC_NHWC, true, 16, 32, false); else FMTC_DECC_F(2, FMTC_NHWC, true, 16, 64, false); }
        else if (log12) {
            if (C == 128) { if (nlo) FMTC_DECC_L(4, FMTC_NHWC, true, 12, 128, true, 2); else FMTC_DECC_L(4, FMTC_NHWC, true, 12, 128, true, 0); }
            else { if (nlo) FMTC_DECC_L(5, FMTC_NHWC, true, 8, 144, true, 3); else FMTC_DECC_L(5, FMTC_NHWC, true, 8, 144, true, 0); }
        }
        else if (ncs == 5) { if (al) FMTC_DECC(5, FMTC_NHWC, true, 4); else FMTC_DECC(5, FMTC_NHWC, false, 4); }
        else if (layout == FMTC_NHWC) { if (al) FMTC_DECC_N(FMTC_NHWC, true); else FMTC_DECC_N(FMTC_NHWC, false); }
        else                          { if (al) FMTC_DECC_N(FMTC_NCHW, true); else FMTC_DECC_N(FMTC_NCHW, false); }
#undef FMTC_DECC_N
#undef FMTC_DECC
#undef FMTC_DECC_F
#undef FMTC_DECC_L
        return el;
    }

    // ---- tiles of several chunks per workgroup ----
    // A workgroup tile is 128 pixels x 256 output channels (4 x 8 matrix tiles), or 64 x 256 for more than 512
    // channels (the symbols of 128 such pixels would not fit LDS): as many chunks as give that many pixels at the
    // nominal chunk size, 16 at most.
    const int n_cg = (ncs + 7) / 8;
    auto chunks_for = [&](int px) {
        int n = (int)(px / (int64_t)g.px_per_chunk);
        return n < 1 ? 1 : (n > 16 ? 16 : n);
    };
    // ... and 64 pixels also where 128 would leave most of the device without a workgroup
    const bool wide = C > 512 || (uint64_t)((g.n_chunks + chunks_for(128) - 1) / chunks_for(128)) * n_cg < 128;
    int G = chunks_for(wide ? 64 : 128);
    if (d_syms) G = 8;  // symbols only: no projection to feed, one chunk per wavefront and as many workgroups as that gives
    p.G = G;
    // the grid is sized from the nominal geometry; the kernel takes the real one from the header
    const uint32_t n_tiles = (g.n_chunks + G - 1) / G;
    // the channel groups (256 channels) of a tile go to workgroups of their own (each decodes the tile's
    // symbols again) while that still fills the device; otherwise a workgroup walks them in turn
    int groups = 1;
    if (!d_syms) {
        groups = (int)(1024 / (n_tiles < 1024u ? n_tiles : 1024u));
        if (groups > n_cg) groups = n_cg;
        if (groups < 1) groups = 1;
        // (a test can make every workgroup walk all channel groups of its tile, as it does for tensors with more
        // tiles than the device holds)
        if (test_option(kTestDecodeOneRow)) groups = 1;
    }
    unsigned gx = n_tiles < 1024u ? n_tiles : 1024u;
    dim3 grid(gx, (unsigned)groups);
    const size_t lds = (size_t)G * 4096 + (size_t)G * 4096 / 16 + 128;
    // more than 64 KB of dynamic LDS has to be requested per kernel (the CU has 160 KB)
#define FMTC_DEC(MT, LAY, AL)                                                                                \
    do {                                                                                                     \
        if (lds > 32 * 1024) {                                                                               \
            hipError_t ea = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_decode_tiles<MT, LAY, AL>), \
                                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);      \
            if (ea != hipSuccess) return ea;                                                                 \
        }                                                                                                    \
        el = launch(K_DECODE, k_decode_tiles<MT, LAY, AL>, grid, dim3(512), lds, s, p);                      \
    } while (0)
    if (layout == FMTC_NHWC) {
        if (al) { if (wide) FMTC_DEC(2, FMTC_NHWC, true); else FMTC_DEC(4, FMTC_NHWC, true); }
        else    { if (wide) FMTC_DEC(2, FMTC_NHWC, false); else FMTC_DEC(4, FMTC_NHWC, false); }
    } else {
        if (al) { if (wide) FMTC_DEC(2, FMTC_NCHW, true); else FMTC_DEC(4, FMTC_NCHW, true); }
        else    { if (wide) FMTC_DEC(2, FMTC_NCHW, false); else FMTC_DEC(4, FMTC_NCHW, false); }
    }
#undef FMTC_DEC
    return el;
}

// Whole decoder of the 8-bit path in one kernel: the chunk decoder with the integer reconstruction in place of the
// f16 one.  *applies = false (and nothing launched) for tensors of more than 128 channels, which the caller then
// decodes to symbols and reconstructs with the tile kernel.
hipError_t launch_decode_u8(const Basis8Device& b, const uint8_t* d_stream, size_t bytes, const Geometry& g, int bits,
                            int64_t HW, int layout, double h, uint8_t* d_xq_hat, uint32_t* d_err, bool* applies,
                            hipStream_t s) {
    const int C = g.C;
    const int ncs = (C + 31) / 32;
    *applies = ncs <= 4;
    if (!*applies) return hipSuccess;
    if (!d_stream || !d_xq_hat || !d_err || !b.inv8 || !b.col_sum || !b.mean_d || b.C != C) return hipErrorInvalidValue;
    DecodeParams p{};
    p.stream = d_stream;
    p.bytes = bytes;
    p.P = g.P;
    p.HW = HW;
    p.C = C;
    p.bits = bits;
    p.ncs = ncs;
    p.Bp16 = nullptr;
    p.mu = nullptr;
    p.xhat = nullptr;
    p.syms_out = nullptr;
    p.err = d_err;
    p.prebuilt = nullptr;
    p.G = 1;
    p.g_off_chunk_off = g.off_chunk_off;
    p.g_off_sub_bits = g.off_sub_bits;
    p.g_off_payload = g.off_payload;
    p.g_n_chunks = g.n_chunks;
    p.g_spc = g.subs_per_chunk;
    p.active_steps = ncs * 2;  // (not used by the 8-bit variant)
    p.op8 = b.inv8;
    p.col_sum = b.col_sum;
    p.mean_d = b.mean_d;
    p.factor8 = h;
    p.out8 = d_xq_hat;
    const bool al = (C % 4) == 0;
    const size_t lds_basis = (size_t)ncs * ((C + 15) / 16) * 64 * 8;  // the basis operand
    const bool eight = g.n_chunks > 1024 && ncs != 3;
    p.lds_basis_bytes = (uint32_t)lds_basis;
    p.pay_words = 128u * (uint32_t)bits + 64u;
    auto lds_dyn = [&](int wv) { return lds_basis + (size_t)wv * (p.pay_words + kPayOverrun) * 4; };
    // four wavefronts per SIMD under the conditions of the fp32 decoder (see launch_decode)
    const bool sixteen = g.n_chunks > 3072 && ncs <= 2 && C == ncs * 32 && layout == FMTC_NHWC &&
                         lds_dyn(16) + sizeof(DecTables) + 16 * (size_t)kChunkTileBytes + 64 <= 160 * 1024;
    const int waves = sixteen ? 16 : (eight ? 8 : 4);
    const size_t lds = lds_dyn(waves);
    unsigned gx = (g.n_chunks + waves - 1) / waves;
    const unsigned cap = 256u * (waves >= 8 ? 1u : 2u);
    if (gx > cap) gx = cap;
    hipError_t el = hipSuccess;
#define FMTC_DECU_F(NCT, LAY, AL, WV, CF) \
    do {                                                                                                         \
        hipError_t ea = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_decode_chunks<NCT, LAY, AL, WV, true, CF>), \
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);              \
        if (ea != hipSuccess) return ea;                                                                         \
        el = launch(K_DECODE, k_decode_chunks<NCT, LAY, AL, WV, true, CF>, dim3(gx), dim3(WV * 64), lds, s, p);  \
    } while (0)
#define FMTC_DECU(NCT, LAY, AL, WV) FMTC_DECU_F(NCT, LAY, AL, WV, 0)
#define FMTC_DECU_N(LAY, AL)                                                                                     \
    do {                                                                                                         \
        if (ncs == 1) { if (eight) FMTC_DECU(1, LAY, AL, 8); else FMTC_DECU(1, LAY, AL, 4); }                    \
        else if (ncs == 2) { if (eight) FMTC_DECU(2, LAY, AL, 8); else FMTC_DECU(2, LAY, AL, 4); }               \
        else if (ncs == 3) FMTC_DECU(3, LAY, AL, 4);                                                             \
        else { if (eight) FMTC_DECU(4, LAY, AL, 8); else FMTC_DECU(4, LAY, AL, 4); }                             \
    } while (0)
    if (sixteen) { if (ncs == 1) FMTC_DECU_F(1, FMTC_NHWC, true, 16, 32); else FMTC_DECU_F(2, FMTC_NHWC, true, 16, 64); }
    else if (layout == FMTC_NHWC) { if (al) FMTC_DECU_N(FMTC_NHWC, true); else FMTC_DECU_N(FMTC_NHWC, false); }
    else                     { if (al) FMTC_DECU_N(FMTC_NCHW, true); else FMTC_DECU_N(FMTC_NCHW, false); }
#undef FMTC_DECU_N
#undef FMTC_DECU
#undef FMTC_DECU_F
    return el;
}

}  // namespace fmtc
