// Internal declarations shared by the host API and the kernel files of libfmtc.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "fmtc.h"

namespace fmtc {

constexpr uint32_t kMagic = 0x43544D46u;  // bytes 'F','M','T','C'
constexpr int kHeaderBytes = 64;
constexpr int kLenTableBytes = 256;
constexpr int kSubSyms = 64;     // symbols per run; one lane codes one run
constexpr int kMaxLen = 48;      // longest code length accepted
constexpr int kMaxHistParts = 1024;  // per-workgroup partial histograms (no atomics, nothing to clear)
constexpr int kLutBits = 11;     // decoder lookup table covers codes up to this length

// 64-byte stream header (see fmtc.h for the field meaning).
struct alignas(8) Header {
    uint32_t magic;
    uint16_t version;
    uint8_t bits;
    uint8_t reserved0;
    uint32_t C;
    uint32_t px_per_chunk;
    uint64_t P;
    uint32_t n_chunks;
    uint32_t sub_syms;
    float delta;
    uint32_t subs_per_chunk;
    uint64_t payload_words;
    uint64_t payload_bits;
    uint64_t reserved1;
};
static_assert(sizeof(Header) == kHeaderBytes, "header must be 64 bytes");

// Where the sections of a container start, from the tensor geometry alone.
struct Geometry {
    int64_t P;
    int C;
    uint32_t px_per_chunk, n_chunks, subs_per_chunk;
    uint32_t chunk_syms;  // px_per_chunk * C
    size_t off_chunk_off, off_sub_bits, off_payload;
};

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

inline bool make_geometry(int64_t P, int C, int chunk_syms, Geometry* g) {
    if (P < 1 || C < 1 || C > 1024 || chunk_syms < 64 || chunk_syms > 4096) return false;
    int64_t ppc = chunk_syms / C;
    if (ppc < 1) ppc = 1;
    int64_t nch = (P + ppc - 1) / ppc;
    if (nch > 0x7fffffff) return false;
    g->P = P;
    g->C = C;
    g->px_per_chunk = (uint32_t)ppc;
    g->n_chunks = (uint32_t)nch;
    g->chunk_syms = (uint32_t)(ppc * C);
    g->subs_per_chunk = (g->chunk_syms + kSubSyms - 1) / kSubSyms;
    g->off_chunk_off = kHeaderBytes + kLenTableBytes;
    g->off_sub_bits = align_up(g->off_chunk_off + 4 * ((size_t)nch + 1), 16);
    g->off_payload = align_up(g->off_sub_bits + 2 * (size_t)nch * g->subs_per_chunk, 16);
    return true;
}

// Control words of one encoder call (in the workspace).  Zeroed by the first kernel of the call.
struct alignas(64) CoderCtrl {
    uint32_t reserved0;
    uint32_t max_len;                 // longest code length (table kernel)
    unsigned long long payload_bits;  // sum of count * length (table kernel)
    uint32_t error;                   // set if a bounded wait of the pack kernel ran out
    uint32_t reserved[11];
};
static_assert(sizeof(CoderCtrl) == 64, "control block is 64 bytes");

constexpr int kPackWaves = 4;  // chunks per workgroup of the pack kernel (one wavefront each)

// Device workspace of the encoder.
struct Workspace {
    size_t off_hist_parts;   // u32 [kMaxHistParts][2^bits] partial histograms, one row per workgroup
    size_t off_ctrl;         // CoderCtrl
    size_t off_hist;         // u32 [256] final histogram
    size_t off_enc_table;    // u64 [256]: bit-reversed code | length << 56
    size_t off_lookback;     // u64 [n_groups]: running payload word count per chunk group (flag << 32 | words)
    size_t off_chunk_bits;   // u32 [n_chunks]: code bits per chunk (tensors packed at precomputed offsets)
    size_t off_syms;         // u8 [V]
    size_t total;
};

inline uint32_t pack_groups(uint32_t n_chunks) { return (n_chunks + kPackWaves - 1) / kPackWaves; }

inline Workspace make_workspace(uint64_t V, uint32_t n_chunks) {
    Workspace w;
    size_t o = 0;
    w.off_hist_parts = o;
    o += sizeof(uint32_t) * kMaxHistParts * 256;
    w.off_ctrl = o;
    o += sizeof(CoderCtrl);
    w.off_hist = o;
    o += sizeof(uint32_t) * 256;
    w.off_enc_table = o;
    o += sizeof(uint64_t) * 256;
    w.off_lookback = o;
    o = align_up(o + sizeof(uint64_t) * (size_t)pack_groups(n_chunks), 256);
    w.off_chunk_bits = o;
    o = align_up(o + sizeof(uint32_t) * (size_t)n_chunks, 256);
    w.off_syms = o;
    o = align_up(o + (size_t)V, 256);
    w.total = o;
    return w;
}

// Device copies of the basis a handle holds.
struct BasisDevice {
    int C, Cpad;           // Cpad = C rounded up to 32
    // M = T and M = T^T as f16 hi/lo pairs in the operand order of the 32x32x16 matrix instruction,
    // [row tile][step j][part][lane][8] (see pack_operand16); fwd16 with permuted rows
    const uint16_t* fwd16;
    const uint16_t* inv16;
    float row_norm;        // largest Euclidean norm of a row of T
    int active_rows;       // rows of T up to the last one that is not all zero (a truncated basis has fewer than C)
    const float* mu;       // [Cpad], zero padded
    const float* T;        // [C][C] row major, unpacked
};

// Path choices a test can force (fmtc_test_option in fmtc.h): both only pick between paths a caller reaches anyway.
enum TestOption { kTestStaticTwoKernels = 0, kTestDecodeOneRow = 1, kTestOptionCount };
int test_option(int which);  // current value (0 unless a test set it)

// ---- optional per-kernel timing (fmtc_profile_* in fmtc.h) ----
// When enabled, a launch carries a pair of events that the runtime attaches to the kernel's own dispatch, so
// the elapsed time is the kernel's start-to-end time on the GPU (no bracket of separate marker commands).
enum KernelId { K_PROJECT = 0, K_HISTOGRAM, K_TABLE, K_PACK, K_DECODE, K_COPY, K_QUANTIZE_U8, K_RECONSTRUCT_U8, K_CHUNK_BITS, K_CHUNK_SCAN, K_COUNT };
bool prof_next(int id, hipEvent_t* start, hipEvent_t* stop);

template <class T>
struct same_as { using type = T; };

template <typename... KArgs>
inline hipError_t launch(int id, void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds, hipStream_t s,
                         typename same_as<KArgs>::type... args) {
    void* ptrs[] = {(void*)&args...};
    hipEvent_t a = nullptr, b = nullptr;
    if (prof_next(id, &a, &b))
        return hipExtLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, lds, s, a, b, 0);
    return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, lds, s);
}

// What the kernels that produce symbols hand to the coder.
struct CoderScratch {
    uint32_t* hist_parts;  // [n_parts][2^bits]
    CoderCtrl* ctrl;
    unsigned long long* lookback;
    uint32_t n_groups;
    uint32_t* chunk_bits;  // [n_chunks]
};

// Device side of the 8-bit basis (fmtc_int8_kernels.hip).  nct = ceil(C / 32) tiles of 32 rows, NS = ceil(C / 16)
// contraction steps; every per-row array is padded to nct * 32 entries.
struct Basis8Device {
    int C;
    const unsigned long long* fwd8;  // [nct][NS][64] Tq, operand order, rows of a tile permuted
    const unsigned long long* inv8;  // [nct][NS][64] Tq^T, the same
    const double* row_off;           // sum_c Tq[k][c] (mean_fix[c] - 256 * 128): an integer, exact in fp64
    const int* col_sum;              // sum_k Tq[k][c]
    const int* mean_fix;             // rne(256 mu[c] / s_x)
    const double* mean_d;            // mean_fix / 256 (exact): the mean in activation units
};
// cs == nullptr: symbols only; else the kernel also clears the coder's scratch and writes one partial histogram per
// workgroup (*n_parts of them), as the fp32 projection kernels do.
hipError_t launch_quantize_u8(const Basis8Device& b, const uint8_t* d_xq, int64_t P, int64_t HW, int layout,
                              int bits, double g, uint8_t* d_syms, const CoderScratch* cs, int* n_parts,
                              hipStream_t s);
hipError_t launch_decode_u8(const Basis8Device& b, const uint8_t* d_stream, size_t bytes, const Geometry& g, int bits,
                            int64_t HW, int layout, double h, uint8_t* d_xq_hat, uint32_t* d_err, bool* applies,
                            hipStream_t s);
hipError_t launch_reconstruct_u8(const Basis8Device& b, const uint8_t* d_syms, int64_t P, int64_t HW, int layout,
                                 int bits, double h, uint8_t* d_xq_hat, hipStream_t s);

// The first kernel of an encoder call clears what the coder kernels after it count in.
__device__ __forceinline__ void zero_coder_scratch(CoderCtrl* ctrl, unsigned long long* lookback, uint32_t n_groups) {
    const size_t nthreads = (size_t)gridDim.x * gridDim.y * blockDim.x;
    const size_t gtid = ((size_t)blockIdx.y * gridDim.x + blockIdx.x) * blockDim.x + threadIdx.x;
    for (size_t i = gtid; i < n_groups; i += nthreads) lookback[i] = 0ull;
    if (gtid < sizeof(CoderCtrl) / 4) reinterpret_cast<uint32_t*>(ctrl)[gtid] = 0u;
}

// ---- kernel launchers (definitions in the *_kernels.hip files) ----
hipError_t launch_project_quantize(const BasisDevice& b, const float* d_x, int64_t N, int64_t HW, int layout,
                                   float delta, int bits, uint8_t* d_syms, const CoderScratch& cs, int* n_parts,
                                   hipStream_t s);

hipError_t launch_histogram(const uint8_t* d_syms, uint64_t V, int bits, const CoderScratch& cs, int* n_parts,
                            hipStream_t s);

// Sum of the partial histograms only (staged quantizer entry point).
hipError_t launch_histogram_sum(const uint32_t* d_hist_parts, int n_parts, int bits, uint32_t* d_hist,
                                hipStream_t s);

hipError_t launch_coder(const uint8_t* d_syms, const Geometry& g, int bits, float delta, const CoderScratch& cs,
                        int n_parts, uint64_t* d_enc_table, uint8_t* d_stream, uint64_t cap_words,
                        uint64_t* d_out_bytes, hipStream_t s);

// Packing with a table fixed beforehand (every symbol of the alphabet has a code).
hipError_t launch_coder_static(const uint8_t* d_syms, const Geometry& g, int bits, float delta, const CoderScratch& cs,
                               const uint64_t* d_enc_table, uint32_t max_len, uint8_t* d_stream, uint64_t cap_words,
                               uint64_t* d_out_bytes, hipStream_t s);
hipError_t launch_table_from_lengths(const uint8_t* d_len_table, int bits, uint64_t* d_enc_table, hipStream_t s);
hipError_t launch_table_from_hist(const uint32_t* d_hist_parts, int n_parts, int bits, uint32_t add_each,
                                  uint64_t* d_enc_table, uint8_t* d_len_table, hipStream_t s);

// d_prebuilt: decode tables made beforehand by launch_build_decode_tables (the stream must carry the same code
// lengths), or NULL: every workgroup builds them from the stream
hipError_t launch_decode(const BasisDevice* b, const uint8_t* d_stream, size_t bytes, const Geometry& g, int bits,
                         int64_t HW, int layout, float* d_xhat, uint8_t* d_syms, uint32_t* d_err, const void* d_prebuilt,
                         hipStream_t s);
hipError_t launch_build_decode_tables(const uint8_t* d_len_table, int bits, void* d_prebuilt, uint32_t* d_ok, hipStream_t s);
size_t prebuilt_decode_tables_bytes();

// d_sum [C] must be zero on entry; d_cov [C*C] is overwritten; d_scratch: fit_moments_scratch_bytes(N * HW, C) bytes
hipError_t launch_fit_moments(const float* d_x, int64_t N, int C, int64_t HW, int layout, double* d_sum,
                              double* d_cov, double* d_scratch, hipStream_t s);
size_t fit_moments_scratch_bytes(int64_t P, int C);
hipError_t launch_fit_range(const float* d_x, int64_t N, int C, int64_t HW, int layout, const float* d_t0,
                            const float* d_mu, double* d_amax, hipStream_t s);
hipError_t launch_fill_zero(uint32_t* d_words, size_t n_words, hipStream_t s);
hipError_t launch_copy(void* d_dst, const void* d_src, size_t bytes, hipStream_t s);

}  // namespace fmtc
