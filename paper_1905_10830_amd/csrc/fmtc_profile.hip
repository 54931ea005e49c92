// Optional per-kernel timing with HIP events recorded on the caller's stream
// around every kernel launch of the library.  Off by default; when off the
// hooks cost one branch.  Used by the benchmark to hold each kernel against its
// roofline.
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
const char* const kNames[K_COUNT] = {"k_clear",    "k_project_quantize", "k_histogram",     "k_huffman_table",
                                     "k_run_bits", "k_pack",             "k_decode_tables", "k_decode"};

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

void prof_mark(int id, bool end, hipStream_t s) {
    if (!g_prof.on) return;
    int& n = g_prof.used[id];
    if (n >= g_prof.cap) return;
    if (!end) {
        (void)hipEventRecord(g_prof.start[id][n], s);
    } else {
        (void)hipEventRecord(g_prof.stop[id][n], s);
        n++;
    }
}

}  // namespace fmtc

extern "C" {

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
