// Optional per-kernel timing: when enabled every kernel launch of the library
// carries a pair of HIP events attached to its own dispatch, so the elapsed time
// is the kernel's start-to-end time on the GPU.  Off by default; when off the
// hook costs one branch.  Used by the benchmark to hold each kernel against its
// roofline.  Also home of two utility kernels (zero fill, yardstick copy).
#include <atomic>
#include <vector>

#include "fmtc_internal.h"

namespace fmtc {

namespace {
struct Profiler {
    bool on = false;
    int cap = 0;
    std::vector<hipEvent_t> start[K_COUNT], stop[K_COUNT];
    int used[K_COUNT] = {0};
};
Profiler g_prof;
const char* const kNames[K_COUNT] = {"k_project_quantize", "k_histogram", "k_huffman_table",
                                     "k_pack",             "k_decode",    "k_copy",
                                     "k_quantize_u8",      "k_reconstruct_u8", "k_chunk_bits",
                                     "k_chunk_scan"};

void release() {
    for (int k = 0; k < K_COUNT; k++) {
        for (hipEvent_t e : g_prof.start[k]) (void)hipEventDestroy(e);
        for (hipEvent_t e : g_prof.stop[k]) (void)hipEventDestroy(e);
        g_prof.start[k].clear();
        g_prof.stop[k].clear();
        g_prof.used[k] = 0;
    }
    g_prof.on = false;
    g_prof.cap = 0;
}
}  // namespace

static std::atomic<int> g_test_option[kTestOptionCount];
int test_option(int which) {
    return (which >= 0 && which < kTestOptionCount) ? g_test_option[which].load(std::memory_order_relaxed) : 0;
}

bool prof_next(int id, hipEvent_t* start, hipEvent_t* stop) {
    if (!g_prof.on) return false;
    int& n = g_prof.used[id];
    if (n >= g_prof.cap) return false;
    *start = g_prof.start[id][n];
    *stop = g_prof.stop[id][n];
    n++;
    return true;
}

// Plain device-to-device copy of known size: the yardstick the memory counters are scaled with.
__global__ __launch_bounds__(256) void k_copy(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n16) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

hipError_t launch_copy(void* d_dst, const void* d_src, size_t bytes, hipStream_t s) {
    const size_t n16 = bytes / 16;
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    if (blocks < 1) blocks = 1;
    return launch(K_COPY, k_copy, dim3((unsigned)blocks), dim3(256), 0, s, static_cast<uint4*>(d_dst),
                  static_cast<const uint4*>(d_src), n16);
}

__global__ void k_fill_zero(uint32_t* __restrict__ w, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) w[i] = 0u;
}

hipError_t launch_fill_zero(uint32_t* d_words, size_t n_words, hipStream_t s) {
    if (n_words == 0) return hipSuccess;
    unsigned blocks = (unsigned)((n_words + 255) / 256);
    hipLaunchKernelGGL(k_fill_zero, dim3(blocks), dim3(256), 0, s, d_words, n_words);
    return hipGetLastError();
}

}  // namespace fmtc

extern "C" {

fmtc_status fmtc_test_option(int option, int value) {
    if (option < 0 || option >= fmtc::kTestOptionCount) return FMTC_EINVAL;
    fmtc::g_test_option[option].store(value, std::memory_order_relaxed);
    return FMTC_OK;
}

fmtc_status fmtc_profile_enable(int max_launches_per_kernel) {
    using namespace fmtc;
    release();
    if (max_launches_per_kernel <= 0) return FMTC_OK;
    for (int k = 0; k < K_COUNT; k++)
        for (int i = 0; i < max_launches_per_kernel; i++) {
            hipEvent_t a, b;
            if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) {
                release();
                return FMTC_EHIP;
            }
            g_prof.start[k].push_back(a);
            g_prof.stop[k].push_back(b);
        }
    g_prof.cap = max_launches_per_kernel;
    g_prof.on = true;
    return FMTC_OK;
}

int fmtc_profile_kernels(void) { return fmtc::K_COUNT; }

const char* fmtc_profile_name(int kernel) {
    return (kernel >= 0 && kernel < fmtc::K_COUNT) ? fmtc::kNames[kernel] : "";
}

fmtc_status fmtc_profile_copy(void* d_dst, const void* d_src, size_t bytes, void* hip_stream) {
    if (!d_dst || !d_src || bytes % 16 != 0 || ((uintptr_t)d_dst | (uintptr_t)d_src) % 16 != 0) return FMTC_EINVAL;
    return fmtc::launch_copy(d_dst, d_src, bytes, (hipStream_t)hip_stream) == hipSuccess ? FMTC_OK : FMTC_EHIP;
}

fmtc_status fmtc_profile_read(int kernel, double* avg_ms, double* min_ms, int* launches) {
    using namespace fmtc;
    if (kernel < 0 || kernel >= K_COUNT || !g_prof.on) return FMTC_EINVAL;
    const int n = g_prof.used[kernel];
    double sum = 0.0, mn = 0.0;
    for (int i = 0; i < n; i++) {
        if (hipEventSynchronize(g_prof.stop[kernel][i]) != hipSuccess) return FMTC_EHIP;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, g_prof.start[kernel][i], g_prof.stop[kernel][i]) != hipSuccess) return FMTC_EHIP;
        sum += ms;
        if (i == 0 || ms < mn) mn = ms;
    }
    if (avg_ms) *avg_ms = n ? sum / n : 0.0;
    if (min_ms) *min_ms = mn;
    if (launches) *launches = n;
    return FMTC_OK;
}

}  // extern "C"
