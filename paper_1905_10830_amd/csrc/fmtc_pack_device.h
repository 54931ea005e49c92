// Device code of the bit packer, shared by the packing kernel and the kernel that projects, quantizes and packs
// in one go.
#pragma once
#include "fmtc_device.h"
#include "fmtc_internal.h"

namespace fmtc {

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
    uint32_t* chunk_bits;        // large tensors: code bits of every chunk (k_chunk_bits -> k_chunk_scan)
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

// Symbols of chunk `ch` (0 past the last chunk).
__device__ __forceinline__ uint32_t chunk_len_of(const PackParams& p, uint32_t ch) {
    if (ch >= p.n_chunks) return 0u;
    const uint64_t c0 = (uint64_t)ch * p.chunk_syms;
    return (uint32_t)((p.V - c0 < p.chunk_syms) ? (p.V - c0) : p.chunk_syms);
}

// The symbols of a chunk: register q of lane l holds symbols 256q + 4l .. + 3 (zero past the chunk's end).
// aligned4: every chunk starts on a 4-byte boundary of the symbols (chunk_syms % 4 == 0).
__device__ __forceinline__ void load_chunk_symbols(const PackParams& p, uint32_t ch, int lane, bool aligned4,
                                                   uint32_t (&w)[16]) {
    const uint32_t clen = chunk_len_of(p, ch);
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
}

// What a workgroup that packs keeps in LDS.
struct PackShared {
    unsigned long long tab[256];                                  // bit-reversed code | length << 56
    __align__(16) uint32_t stage[kPackWaves][kStageWords + 4];    // per wavefront: chunk image + the spare words
    uint16_t runs[kPackWaves][64];                                // bit counts of a chunk's runs on their way out
    uint32_t wave_words[kPackWaves], wave_slack[kPackWaves];
    uint32_t excl, excl_slack, max_len;
    unsigned long long payload_bits;
};

// This wavefront's image starts out clear (and whoever reads a word out clears it again).
__device__ __forceinline__ void pack_clear_image(PackShared& S, int wave, int lane) {
    uint32_t* img = S.stage[wave];
    for (int i = lane; i < kStageWords / 4; i += 64) reinterpret_cast<uint4*>(img)[i] = make_uint4(0u, 0u, 0u, 0u);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// One group of kPackWaves chunks, chunk group * kPackWaves + wavefront in each wavefront: `w` holds its `clen`
// symbols (register q of lane l: symbols 256q + 4l .. + 3, zero past the chunk's end; clen = 0 past the last
// chunk).  Called by all 256 threads; contains workgroup barriers.  `between` runs once in every thread after the
// group's size is published and before the wait for its position: the place to start loads for the next group.
template <int MODE, class Between>
__device__ __forceinline__ void pack_group(PackShared& S, const PackParams& p, uint32_t group, const uint32_t (&w)[16],
                                           uint32_t clen, Between&& between) {
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wavefront-uniform by construction
    const uint32_t max_len = S.max_len;
    uint32_t* img = S.stage[wave];
    uint16_t* sub_bits = reinterpret_cast<uint16_t*>(p.stream + p.off_sub_bits);
    uint32_t* chunk_off = reinterpret_cast<uint32_t*>(p.stream + kHeaderBytes + kLenTableBytes);
    const uint32_t ch = group * kPackWaves + (uint32_t)wave;
    const bool have = ch < p.n_chunks;
    auto wave_sync = [&]() {
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    };

    // ---- the first window of the chunk's image: needs no global position ----
    // (the image is all zero here: cleared once at the start and again by whoever reads a word out)
    auto build_window = [&](uint32_t win, uint32_t win_words, uint16_t* run_bits) -> uint32_t {
        uint32_t total;
        const uint32_t n_runs = p.subs_per_chunk;
        if (win == 0) {
            if (max_len <= 32) total = pack_chunk<false, true>(w, clen, S.tab, img, win, win_words, lane, run_bits, n_runs);
            else total = pack_chunk<true, true>(w, clen, S.tab, img, win, win_words, lane, run_bits, n_runs);
        } else {
            if (max_len <= 32) total = pack_chunk<false, false>(w, clen, S.tab, img, win, win_words, lane, run_bits, n_runs);
            else total = pack_chunk<true, false>(w, clen, S.tab, img, win, win_words, lane, run_bits, n_runs);
        }
        wave_sync();  // the ORs of all lanes precede the reads that follow
        return total;
    };
    uint32_t n_words = 0, slack = 0;
    if (have) {
        // the run sizes are produced four at a time: up to 64 of them are collected in LDS and leave as one
        // contiguous store (scattered two-byte stores cost a partial memory write each)
        uint16_t* runs_out = sub_bits + (size_t)ch * p.subs_per_chunk;
        const bool staged = p.subs_per_chunk <= 64u;
        const uint32_t total_bits = build_window(0, kStageWords, staged ? S.runs[wave] : runs_out);
        if (staged && (uint32_t)lane < p.subs_per_chunk) runs_out[lane] = S.runs[wave][lane];
        n_words = (total_bits + 31) >> 5;
        slack = 32u * n_words - total_bits;
    }
    if (lane == 0) {
        S.wave_words[wave] = n_words;
        S.wave_slack[wave] = slack;
    }
    __syncthreads();
    uint32_t agg = 0, agg_slack = 0;
#pragma unroll
    for (int q = 0; q < kPackWaves; q++) {
        agg += S.wave_words[q];
        agg_slack += S.wave_slack[q];
    }
    if (tid == 0)
        publish64(&p.lookback[group], (group == 0 ? kFlagInclusive : kFlagAggregate) |
                                          ((unsigned long long)agg_slack << 32) | agg);

    between();

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
            if (lane == 0) __hip_atomic_fetch_or(&p.ctrl->error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            excl = 0;
            excl_slack = 0;
        }
        if (lane == 0) {
            publish64(&p.lookback[group], kFlagInclusive | ((unsigned long long)(excl_slack + agg_slack) << 32) |
                                              (unsigned long long)(excl + agg));
            S.excl = excl;
            S.excl_slack = excl_slack;
        }
    } else if (tid == 0) {
        S.excl = 0;
        S.excl_slack = 0;
    }
    __syncthreads();
    if (have) {
        uint32_t word0 = S.excl;
        for (int q = 0; q < wave; q++) word0 += S.wave_words[q];
        if (lane == 0) {
            chunk_off[ch] = word0;
            if (ch == p.n_chunks - 1) {
                const uint64_t total_words = (uint64_t)word0 + n_words;
                chunk_off[p.n_chunks] = (uint32_t)total_words;
                Header hdr = p.hdr;
                hdr.payload_words = total_words;
                hdr.payload_bits = S.payload_bits;
                if constexpr (MODE == kPackStatic) {
                    // every code bit of the tensor: the words of all chunks less what their last words leave unused
                    uint32_t total_slack = S.excl_slack + slack;
                    for (int q = 0; q < wave; q++) total_slack += S.wave_slack[q];
                    hdr.payload_bits = 32ull * total_words - total_slack;
                }
                // a wait gave up, or the payload outgrew the buffer (then some chunk was not written): not valid
                if (__hip_atomic_load(&p.ctrl->error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) || total_words > p.cap_words) hdr.magic = 0u;
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
        // histogram and the symbols ever disagree, or a table made beforehand not fit the tensor, nothing is
        // written past the buffer: the stream is marked invalid instead.)
        const bool fits = (uint64_t)word0 + n_words <= p.cap_words;
        if (!fits && lane == 0) __hip_atomic_fetch_or(&p.ctrl->error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
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
    __syncthreads();  // wave_words, wave_slack and excl* are rewritten by the next group
}

// Host side (fmtc_coder_kernels.hip): the packer's arguments for a tensor geometry.
PackParams pack_params(const uint8_t* d_syms, const Geometry& g, int bits, float delta, const CoderScratch& cs,
                       int n_parts, const uint64_t* d_enc_table, uint8_t* d_stream, uint64_t cap_words,
                       uint64_t* d_out_bytes);
bool encode_static_fused_applies(int C, int layout, uint32_t chunk_syms, uint32_t n_groups);
hipError_t launch_encode_static_fused(const BasisDevice& b, const float* d_x, int64_t N, int64_t HW, int layout,
                                      float delta, int bits, const CoderScratch& cs, const PackParams& pk,
                                      hipStream_t s);

}  // namespace fmtc
