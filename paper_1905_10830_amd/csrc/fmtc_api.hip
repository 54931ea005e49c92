// Host side of libfmtc: argument checks, the basis handle, the offline fit and
// the launch sequences of the encoder and decoder.  See include/fmtc.h.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <atomic>
#include <cstring>
#include <new>
#include <vector>

#include "fmtc_internal.h"
#include "fmtc_pack_device.h"

struct fmtc_basis {
    int C = 0, Cpad = 0;
    float range_A = 0.f;
    std::vector<float> T, mu;
    std::vector<double> eig;
    float *d_mu = nullptr, *d_T = nullptr;
    uint16_t *d_fwd16 = nullptr, *d_inv16 = nullptr;
    float row_norm = 1.f;  // largest Euclidean norm of a row of T (1 for an orthonormal basis)
    int active_rows = 0;   // rows up to the last one that is not all zero
    int device = 0;
};

struct fmtc_table {
    int bits = 0;
    uint32_t max_len = 0;
    uint8_t lengths[256] = {0};
    uint64_t* d_enc_table = nullptr;  // [256]: bit-reversed code | length << 56
    void* d_dec_tables = nullptr;     // the decoder's tables for this code, made once
    int device = 0;
};

struct fmtc_basis8 {
    int C = 0;
    float scale_T = 1.f, act_scale = 1.f, range_A = 0.f;
    std::vector<int8_t> Tq;         // [C][C]
    std::vector<int32_t> mean_fix;  // [C]
    void* d_block = nullptr;        // one allocation: fwd8, inv8, row_off, col_sum, mean_fix
    fmtc::Basis8Device view{};
    int device = 0;
};

static __device__ __align__(256) unsigned char scratch[FMTC_NOALLOC_SCRATCH_BYTES];

namespace {

using namespace fmtc;

thread_local char g_err[256] = "";

fmtc_status fail(fmtc_status st, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return st;
}

fmtc_status hip_fail(hipError_t e, const char* what) {
    return fail(FMTC_EHIP, "%s: %s", what, hipGetErrorString(e));
}

// Scratch of fmtc_encode_noalloc: the encoder's workspace as a device array that lives in the library's code
// object, one copy per GPU, held until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress: the address a kernel may use is resolved once per device (with that device current) and
// kept here; host code never passes the name itself to a kernel or a copy.
constexpr size_t kNoAllocScratchBytes = FMTC_NOALLOC_SCRATCH_BYTES;
constexpr int kNoAllocMaxDevices = 64;
std::atomic<uint8_t*> g_noalloc_scratch_ptr[kNoAllocMaxDevices];

// Runs the body of an entry point that allocates host memory; an allocation failure comes back as a status (nothing
// may be thrown across the C boundary).
template <class F>
fmtc_status guarded(F&& body) {
    try {
        return body();
    } catch (const std::bad_alloc&) {
        return fail(FMTC_ENOMEM, "host allocation failed");
    } catch (...) {
        return fail(FMTC_EHIP, "unexpected failure inside the library");
    }
}

bool dims_ok(int64_t N, int C, int H, int W) {
    if (N < 1 || C < 1 || C > 1024 || H < 1 || W < 1) return false;
    long double v = (long double)N * C * H * W;
    return v < 4294967296.0L;
}

bool aligned(const void* p, size_t a) { return ((uintptr_t)p % a) == 0; }

// Operand order of the kernels (v_mfma_f32_32x32x16_f16, every fp32 entry split into two f16 parts:
// hi = the entry rounded to f16, lo = 2^11 times the rest, rounded to f16).  For tile t (32 rows of M) and step
// j (16 columns) the 64 lanes' hi parts (8 halves each) are followed by their lo parts:
//   out[(((t * NJ + j) * 2 + part) * 64 + lane) * 8 + e] = part of M[t*32 + row(lane%32)][16j + 8*(lane/32) + e],
// NJ = Cpad / 16, zero outside CxC.  With permute_rows the rows of a tile are taken in the order that leaves a
// lane of the matrix instruction with 16 consecutive rows.
void pack_operand16(const std::vector<float>& T, int C, int Cpad, bool transpose, bool permute_rows,
                    std::vector<uint16_t>* out) {
    const int nt_count = Cpad / 32, NJ = Cpad / 16;
    out->assign((size_t)2 * Cpad * Cpad, 0);
    for (int nt = 0; nt < nt_count; nt++)
        for (int j = 0; j < NJ; j++)
            for (int lane = 0; lane < 64; lane++)
                for (int e = 0; e < 8; e++) {
                    const int r = lane % 32, half = lane / 32;
                    const int row = nt * 32 + (permute_rows ? 16 * ((r >> 2) & 1) + 4 * (r >> 3) + (r & 3) : r);
                    const int col = 16 * j + 8 * half + e;
                    float v = 0.f;
                    if (row < C && col < C) v = transpose ? T[(size_t)col * C + row] : T[(size_t)row * C + col];
                    const _Float16 hi = (_Float16)v;
                    const _Float16 lo = (_Float16)((v - (float)hi) * 2048.f);
                    uint16_t hb, lb;
                    memcpy(&hb, &hi, 2);
                    memcpy(&lb, &lo, 2);
                    const size_t base = ((size_t)nt * NJ + j) * 2;
                    (*out)[((base + 0) * 64 + lane) * 8 + e] = hb;
                    (*out)[((base + 1) * 64 + lane) * 8 + e] = lb;
                }
}

fmtc_status upload_basis(fmtc_basis* b) {
    const int C = b->C, Cpad = b->Cpad;
    std::vector<float> mu(Cpad, 0.f);
    std::vector<uint16_t> fwd16, inv16;
    pack_operand16(b->T, C, Cpad, false, true, &fwd16);
    pack_operand16(b->T, C, Cpad, true, false, &inv16);
    double worst = 0.0;
    for (int k = 0; k < C; k++) {
        double n2 = 0.0;
        for (int c = 0; c < C; c++) n2 += (double)b->T[(size_t)k * C + c] * (double)b->T[(size_t)k * C + c];
        if (n2 > worst) worst = n2;
    }
    b->row_norm = (float)std::sqrt(worst);
    b->active_rows = 1;
    for (int k = 0; k < C; k++)
        for (int c = 0; c < C; c++)
            if (b->T[(size_t)k * C + c] != 0.f) { b->active_rows = k + 1; break; }
    for (int c = 0; c < C; c++) mu[c] = b->mu[c];
    hipError_t e;
    const size_t mat = sizeof(float) * (size_t)Cpad * Cpad;
    if ((e = hipGetDevice(&b->device)) != hipSuccess) return hip_fail(e, "hipGetDevice");
    if ((e = hipMalloc((void**)&b->d_mu, sizeof(float) * Cpad)) != hipSuccess) return fail(FMTC_ENOMEM, "hipMalloc basis: %s", hipGetErrorString(e));
    if ((e = hipMemcpy(b->d_mu, mu.data(), sizeof(float) * Cpad, hipMemcpyHostToDevice)) != hipSuccess) return hip_fail(e, "hipMemcpy basis");
    if ((e = hipMalloc((void**)&b->d_inv16, mat)) != hipSuccess) return fail(FMTC_ENOMEM, "hipMalloc basis: %s", hipGetErrorString(e));
    if ((e = hipMemcpy(b->d_inv16, inv16.data(), mat, hipMemcpyHostToDevice)) != hipSuccess) return hip_fail(e, "hipMemcpy basis");
    if ((e = hipMalloc((void**)&b->d_fwd16, mat)) != hipSuccess) return fail(FMTC_ENOMEM, "hipMalloc basis: %s", hipGetErrorString(e));
    if ((e = hipMemcpy(b->d_fwd16, fwd16.data(), mat, hipMemcpyHostToDevice)) != hipSuccess) return hip_fail(e, "hipMemcpy basis");
    if ((e = hipMalloc((void**)&b->d_T, sizeof(float) * (size_t)C * C)) != hipSuccess) return fail(FMTC_ENOMEM, "hipMalloc basis: %s", hipGetErrorString(e));
    if ((e = hipMemcpy(b->d_T, b->T.data(), sizeof(float) * (size_t)C * C, hipMemcpyHostToDevice)) != hipSuccess) return hip_fail(e, "hipMemcpy basis");
    return FMTC_OK;
}

BasisDevice device_view(const fmtc_basis* b) {
    BasisDevice v;
    v.C = b->C;
    v.Cpad = b->Cpad;
    v.inv16 = b->d_inv16;
    v.fwd16 = b->d_fwd16;
    v.row_norm = b->row_norm;
    v.active_rows = b->active_rows;
    v.mu = b->d_mu;
    v.T = b->d_T;
    return v;
}

// Eigenvalues and eigenvectors of a symmetric matrix by threshold Jacobi
// rotations on rows (the matrix and the accumulated rotations are kept so that
// every update runs over contiguous memory).  a: n*n, overwritten; vt: n*n, row i
// becomes the eigenvector of eigenvalue a[i][i].
void symmetric_eigen(std::vector<double>& a, std::vector<double>& vt, int n) {
    vt.assign((size_t)n * n, 0.0);
    for (int i = 0; i < n; i++) vt[(size_t)i * n + i] = 1.0;
    double total = 0.0;
    for (double v : a) total += v * v;
    if (total == 0.0) return;
    for (int sweep = 0; sweep < 60; sweep++) {
        double off = 0.0;
        for (int p = 0; p < n; p++)
            for (int q = p + 1; q < n; q++) off += a[(size_t)p * n + q] * a[(size_t)p * n + q];
        if (2.0 * off <= 1e-28 * total) break;
        for (int p = 0; p < n - 1; p++) {
            double* ap = &a[(size_t)p * n];
            for (int q = p + 1; q < n; q++) {
                double* aq = &a[(size_t)q * n];
                const double apq = ap[q];
                if (apq == 0.0) continue;
                const double diff = aq[q] - ap[p];
                double t;
                if (std::fabs(apq) < 1e-300 * std::fabs(diff)) {
                    t = apq / diff;
                } else {
                    const double theta = 0.5 * diff / apq;
                    t = 1.0 / (std::fabs(theta) + std::sqrt(theta * theta + 1.0));
                    if (theta < 0.0) t = -t;
                }
                const double c = 1.0 / std::sqrt(t * t + 1.0), s = t * c;
                const double app = ap[p], aqq = aq[q];
                // rows p and q of A, then the two columns by symmetry
                for (int k = 0; k < n; k++) {
                    const double x = ap[k], y = aq[k];
                    ap[k] = c * x - s * y;
                    aq[k] = s * x + c * y;
                }
                ap[p] = app - t * apq;
                aq[q] = aqq + t * apq;
                ap[q] = 0.0;
                aq[p] = 0.0;
                for (int k = 0; k < n; k++) {
                    if (k == p || k == q) continue;
                    a[(size_t)k * n + p] = ap[k];
                    a[(size_t)k * n + q] = aq[k];
                }
                double* vp = &vt[(size_t)p * n];
                double* vq = &vt[(size_t)q * n];
                for (int k = 0; k < n; k++) {
                    const double x = vp[k], y = vq[k];
                    vp[k] = c * x - s * y;
                    vq[k] = s * x + c * y;
                }
            }
        }
    }
}

struct EncodePlan {
    Geometry g;
    Workspace ws;
    uint64_t V;
};

fmtc_status plan_encode(int64_t P, int C, int bits, int chunk_syms, EncodePlan* pl) {
    if (bits < 2 || bits > 8) return fail(FMTC_EINVAL, "bits must be in [2,8], got %d", bits);
    if (!make_geometry(P, C, chunk_syms, &pl->g))
        return fail(FMTC_EINVAL, "bad geometry: P=%lld C=%d chunk_syms=%d", (long long)P, C, chunk_syms);
    long double v = (long double)P * C;
    if (v >= 4294967296.0L) return fail(FMTC_EINVAL, "tensor too large: V must be < 2^32");
    pl->V = (uint64_t)P * (uint64_t)C;
    pl->ws = make_workspace(pl->V, pl->g.n_chunks);
    return FMTC_OK;
}

size_t bound_from(const EncodePlan& pl, int bits) {
    return pl.g.off_payload + 4 * (size_t)((pl.V * (uint64_t)bits + 31) / 32 + pl.g.n_chunks);
}

CoderScratch coder_scratch(uint8_t* ws, const EncodePlan& pl) {
    CoderScratch cs;
    cs.hist_parts = reinterpret_cast<uint32_t*>(ws + pl.ws.off_hist_parts);
    cs.ctrl = reinterpret_cast<CoderCtrl*>(ws + pl.ws.off_ctrl);
    cs.lookback = reinterpret_cast<unsigned long long*>(ws + pl.ws.off_lookback);
    cs.n_groups = pack_groups(pl.g.n_chunks);
    cs.chunk_bits = reinterpret_cast<uint32_t*>(ws + pl.ws.off_chunk_bits);
    return cs;
}

// partial histograms -> table -> run sizes, chunk offsets and payload
fmtc_status run_coder(const uint8_t* d_syms, const EncodePlan& pl, const CoderScratch& cs, int n_parts, int bits,
                      float delta, uint8_t* ws, uint8_t* d_stream, size_t cap, uint64_t* d_out_bytes, hipStream_t s) {
    uint64_t* enc_table = reinterpret_cast<uint64_t*>(ws + pl.ws.off_enc_table);
    const uint64_t cap_words = cap > pl.g.off_payload ? (cap - pl.g.off_payload) / 4 : 0;
    hipError_t e = launch_coder(d_syms, pl.g, bits, delta, cs, n_parts, enc_table, d_stream, cap_words, d_out_bytes, s);
    if (e != hipSuccess) return hip_fail(e, "coder kernels");
    return FMTC_OK;
}


// Sums [C] and cross-product sums about this tensor's own mean [C*C] (fp64 matrix cores; 64 x 64 blocks off the
// diagonal are computed once and mirrored, the blocks on it in full: made exactly symmetric here), in fp64.
// Synchronises the stream.
fmtc_status device_moments(const float* d_x, int64_t N, int C, int64_t HW, int layout, hipStream_t s,
                           std::vector<double>* sum, std::vector<double>* m2) {
    hipError_t e;
    double *d_stat = nullptr, *d_part = nullptr;
    const size_t n_stat = (size_t)C + (size_t)C * C;
    if ((e = hipMalloc((void**)&d_stat, sizeof(double) * n_stat)) != hipSuccess ||
        (e = hipMalloc((void**)&d_part, fit_moments_scratch_bytes(N * HW, C))) != hipSuccess) {
        if (d_stat) (void)hipFree(d_stat);
        return fail(FMTC_ENOMEM, "hipMalloc fit scratch: %s", hipGetErrorString(e));
    }
    std::vector<double> stat(n_stat);
    fmtc_status st = FMTC_OK;
    do {
        if ((e = launch_fill_zero(reinterpret_cast<uint32_t*>(d_stat), 2 * (size_t)C, s)) != hipSuccess) { st = hip_fail(e, "clear"); break; }
        if ((e = launch_fit_moments(d_x, N, C, HW, layout, d_stat, d_stat + C, d_part, s)) != hipSuccess) { st = hip_fail(e, "fit moments"); break; }
        if ((e = hipMemcpyAsync(stat.data(), d_stat, sizeof(double) * n_stat, hipMemcpyDeviceToHost, s)) != hipSuccess) { st = hip_fail(e, "copy moments"); break; }
        if ((e = hipStreamSynchronize(s)) != hipSuccess) { st = hip_fail(e, "fit sync"); break; }
    } while (0);
    (void)hipFree(d_stat);
    (void)hipFree(d_part);
    if (st != FMTC_OK) return st;
    sum->assign(stat.begin(), stat.begin() + C);
    m2->assign(stat.begin() + C, stat.end());
    for (int i = 0; i < C; i++)
        for (int j = i + 1; j < C; j++) {
            double m = 0.5 * ((*m2)[(size_t)i * C + j] + (*m2)[(size_t)j * C + i]);
            (*m2)[(size_t)i * C + j] = (*m2)[(size_t)j * C + i] = m;
        }
    return FMTC_OK;
}

// Basis of a mean and a (symmetric) covariance: eigenvectors by descending eigenvalue, each signed so that its
// largest-magnitude entry is positive, rounded to fp32; then A = max |y_0| over the pixels of d_x with the rounded
// leading row and mean, and the upload.  Synchronises the stream.
fmtc_status finish_fit(int C, const std::vector<double>& mean, std::vector<double> cov, const float* d_x, int64_t N,
                       int64_t HW, int layout, hipStream_t s, fmtc_basis** out) {
    std::vector<double> vt;
    symmetric_eigen(cov, vt, C);
    std::vector<int> order(C);
    for (int i = 0; i < C; i++) order[i] = i;
    for (int i = 1; i < C; i++) {  // stable, descending eigenvalue
        int o = order[i], j = i - 1;
        double ev = cov[(size_t)o * C + o];
        while (j >= 0 && cov[(size_t)order[j] * C + order[j]] < ev) { order[j + 1] = order[j]; j--; }
        order[j + 1] = o;
    }
    fmtc_basis* b = new (std::nothrow) fmtc_basis;
    if (!b) return fail(FMTC_ENOMEM, "host allocation failed");
    b->C = C;
    b->Cpad = (C + 31) / 32 * 32;
    b->T.resize((size_t)C * C);
    b->mu.resize(C);
    b->eig.resize(C);
    for (int k = 0; k < C; k++) {
        const double* v = &vt[(size_t)order[k] * C];
        b->eig[k] = cov[(size_t)order[k] * C + order[k]];
        int arg = 0;
        for (int c = 1; c < C; c++)
            if (std::fabs(v[c]) > std::fabs(v[arg])) arg = c;
        const double sgn = v[arg] < 0.0 ? -1.0 : 1.0;
        for (int c = 0; c < C; c++) b->T[(size_t)k * C + c] = (float)(sgn * v[c]);
    }
    for (int c = 0; c < C; c++) b->mu[c] = (float)mean[c];
    hipError_t e;
    fmtc_status st = FMTC_OK;
    float* d_row = nullptr;  // [C] leading row, [C] mean, then the fp64 maximum
    do {
        if ((e = hipMalloc((void**)&d_row, sizeof(float) * 2 * C + 16)) != hipSuccess) { st = fail(FMTC_ENOMEM, "hipMalloc: %s", hipGetErrorString(e)); break; }
        float* d_mu = d_row + C;
        double* d_amax = reinterpret_cast<double*>(reinterpret_cast<uint8_t*>(d_row) + (sizeof(float) * 2 * C + 7) / 8 * 8);
        if ((e = hipMemcpyAsync(d_row, b->T.data(), sizeof(float) * C, hipMemcpyHostToDevice, s)) != hipSuccess) { st = hip_fail(e, "copy"); break; }
        if ((e = hipMemcpyAsync(d_mu, b->mu.data(), sizeof(float) * C, hipMemcpyHostToDevice, s)) != hipSuccess) { st = hip_fail(e, "copy"); break; }
        if ((e = launch_fill_zero(reinterpret_cast<uint32_t*>(d_amax), 2, s)) != hipSuccess) { st = hip_fail(e, "clear"); break; }
        if ((e = launch_fit_range(d_x, N, C, HW, layout, d_row, d_mu, d_amax, s)) != hipSuccess) { st = hip_fail(e, "fit range"); break; }
        double amax = 0.0;
        if ((e = hipMemcpyAsync(&amax, d_amax, sizeof(double), hipMemcpyDeviceToHost, s)) != hipSuccess) { st = hip_fail(e, "copy"); break; }
        if ((e = hipStreamSynchronize(s)) != hipSuccess) { st = hip_fail(e, "fit sync"); break; }
        b->range_A = (float)amax;
        st = upload_basis(b);
    } while (0);
    if (d_row) (void)hipFree(d_row);
    if (st != FMTC_OK) {
        fmtc_basis_destroy(b);
        return st;
    }
    *out = b;
    return FMTC_OK;
}


// Tq or its transpose in the operand order of the integer matrix instruction: for tile t (32 rows), step j (16
// columns) lane l holds the 8 bytes M[32 t + perm(l % 32)][16 j + 8 (l / 32) + e], perm as in pack_operand16.
void pack_operand8(const std::vector<int8_t>& Tq, int C, bool transpose, std::vector<unsigned long long>* out) {
    const int nct = (C + 31) / 32, NS = (C + 15) / 16;
    out->assign((size_t)nct * NS * 64, 0ull);
    for (int t = 0; t < nct; t++)
        for (int j = 0; j < NS; j++)
            for (int lane = 0; lane < 64; lane++) {
                const int r = lane % 32, half = lane / 32;
                const int row = t * 32 + 16 * ((r >> 2) & 1) + 4 * (r >> 3) + (r & 3);
                unsigned long long v = 0ull;
                for (int e = 0; e < 8; e++) {
                    const int col = 16 * j + 8 * half + e;
                    int8_t b = 0;
                    if (row < C && col < C) b = transpose ? Tq[(size_t)col * C + row] : Tq[(size_t)row * C + col];
                    v |= (unsigned long long)(uint8_t)b << (8 * e);
                }
                (*out)[((size_t)t * NS + j) * 64 + lane] = v;
            }
}

fmtc_status upload_basis8(fmtc_basis8* b) {
    const int C = b->C, nct = (C + 31) / 32, NS = (C + 15) / 16, rows = nct * 32;
    std::vector<unsigned long long> fwd, inv;
    pack_operand8(b->Tq, C, false, &fwd);
    pack_operand8(b->Tq, C, true, &inv);
    std::vector<long long> off64(rows, 0);
    std::vector<double> row_off(rows, 0.0);
    std::vector<int> col_sum(rows, 0), mean_fix(rows, 0);
    for (int k = 0; k < C; k++)
        for (int c = 0; c < C; c++) {
            const long long t = b->Tq[(size_t)k * C + c];
            off64[k] += t * ((long long)b->mean_fix[c] - 256ll * 128ll);
            col_sum[c] += (int)t;
        }
    // |off| <= 127 * 1024 * 2^30 < 2^48: exact as a double
    for (int k = 0; k < C; k++) row_off[k] = (double)off64[k];
    for (int c = 0; c < C; c++) mean_fix[c] = b->mean_fix[c];
    std::vector<double> mean_d(rows, 0.0);
    for (int c = 0; c < C; c++) mean_d[c] = (double)b->mean_fix[c] / 256.0;
    const size_t n_op = (size_t)nct * NS * 64 * sizeof(unsigned long long);
    const size_t o_inv = n_op, o_off = 2 * n_op, o_col = o_off + sizeof(double) * rows,
                 o_mean = o_col + sizeof(int) * rows, o_meand = (o_mean + sizeof(int) * rows + 7) / 8 * 8,
                 total = o_meand + sizeof(double) * rows;
    hipError_t e;
    if ((e = hipGetDevice(&b->device)) != hipSuccess) return hip_fail(e, "hipGetDevice");
    if ((e = hipMalloc(&b->d_block, total)) != hipSuccess) return fail(FMTC_ENOMEM, "hipMalloc basis: %s", hipGetErrorString(e));
    uint8_t* d = static_cast<uint8_t*>(b->d_block);
    if ((e = hipMemcpy(d, fwd.data(), n_op, hipMemcpyHostToDevice)) != hipSuccess ||
        (e = hipMemcpy(d + o_inv, inv.data(), n_op, hipMemcpyHostToDevice)) != hipSuccess ||
        (e = hipMemcpy(d + o_off, row_off.data(), sizeof(double) * rows, hipMemcpyHostToDevice)) != hipSuccess ||
        (e = hipMemcpy(d + o_col, col_sum.data(), sizeof(int) * rows, hipMemcpyHostToDevice)) != hipSuccess ||
        (e = hipMemcpy(d + o_mean, mean_fix.data(), sizeof(int) * rows, hipMemcpyHostToDevice)) != hipSuccess ||
        (e = hipMemcpy(d + o_meand, mean_d.data(), sizeof(double) * rows, hipMemcpyHostToDevice)) != hipSuccess)
        return hip_fail(e, "hipMemcpy basis");
    b->view.C = C;
    b->view.fwd8 = reinterpret_cast<const unsigned long long*>(d);
    b->view.inv8 = reinterpret_cast<const unsigned long long*>(d + o_inv);
    b->view.row_off = reinterpret_cast<const double*>(d + o_off);
    b->view.col_sum = reinterpret_cast<const int*>(d + o_col);
    b->view.mean_fix = reinterpret_cast<const int*>(d + o_mean);
    b->view.mean_d = reinterpret_cast<const double*>(d + o_meand);
    return FMTC_OK;
}

}  // namespace

extern "C" {

const char* fmtc_last_error(void) { return g_err; }

float fmtc_delta(float range_A, int bits) {
    if (!(range_A > 0.0f) || bits < 2 || bits > 8) return 1.0f;
    return (float)((double)range_A / (double)((1 << (bits - 1)) - 1));
}

int fmtc_basis_channels(const fmtc_basis* basis) { return basis ? basis->C : 0; }

void fmtc_basis_destroy(fmtc_basis* b) {
    if (!b) return;
    if (b->d_inv16) (void)hipFree(b->d_inv16);
    if (b->d_fwd16) (void)hipFree(b->d_fwd16);
    if (b->d_mu) (void)hipFree(b->d_mu);
    if (b->d_T) (void)hipFree(b->d_T);
    delete b;
}

fmtc_status fmtc_basis_import(int C, const float* h_T, const float* h_mu, float range_A, fmtc_basis** out) {
    return guarded([&]() -> fmtc_status {
    if (!out) return fail(FMTC_EINVAL, "out is NULL");
    *out = nullptr;
    if (C < 1 || C > 1024 || !h_T || !h_mu) return fail(FMTC_EINVAL, "bad basis arguments (C=%d)", C);
    if (!(range_A >= 0.f)) return fail(FMTC_EINVAL, "range_A must be >= 0");
    fmtc_basis* b = new (std::nothrow) fmtc_basis;
    if (!b) return fail(FMTC_ENOMEM, "host allocation failed");
    b->C = C;
    b->Cpad = (C + 31) / 32 * 32;
    b->range_A = range_A;
    b->T.assign(h_T, h_T + (size_t)C * C);
    b->mu.assign(h_mu, h_mu + C);
    b->eig.assign(C, 0.0);
    fmtc_status st = upload_basis(b);
    if (st != FMTC_OK) {
        fmtc_basis_destroy(b);
        return st;
    }
    *out = b;
    return FMTC_OK;
    });
}

fmtc_status fmtc_basis_export(const fmtc_basis* b, float* h_T, float* h_mu, double* h_eigvals, float* range_A) {
    if (!b) return fail(FMTC_EINVAL, "basis is NULL");
    if (h_T) memcpy(h_T, b->T.data(), sizeof(float) * b->T.size());
    if (h_mu) memcpy(h_mu, b->mu.data(), sizeof(float) * b->mu.size());
    if (h_eigvals) memcpy(h_eigvals, b->eig.data(), sizeof(double) * b->eig.size());
    if (range_A) *range_A = b->range_A;
    return FMTC_OK;
}

fmtc_status fmtc_fit_basis(const float* d_x, int64_t N, int C, int H, int W, fmtc_layout layout, void* hip_stream,
                           fmtc_basis** out) {
    return guarded([&]() -> fmtc_status {
    if (!out) return fail(FMTC_EINVAL, "out is NULL");
    *out = nullptr;
    if (!d_x || !dims_ok(N, C, H, W)) return fail(FMTC_EINVAL, "bad tensor arguments");
    if (layout != FMTC_NCHW && layout != FMTC_NHWC) return fail(FMTC_EINVAL, "bad layout");
    hipStream_t s = (hipStream_t)hip_stream;
    const int64_t HW = (int64_t)H * W, P = N * HW;
    std::vector<double> sum, m2;
    fmtc_status st = device_moments(d_x, N, C, HW, layout, s, &sum, &m2);
    if (st != FMTC_OK) return st;
    std::vector<double> mean(C);
    for (int c = 0; c < C; c++) mean[c] = sum[c] / (double)P;
    for (size_t i = 0; i < m2.size(); i++) m2[i] /= (double)P;
    return finish_fit(C, mean, m2, d_x, N, HW, layout, s, out);
    });
}

struct fmtc_fit_state {
    int C = 0;
    int64_t count = 0;            // pixels seen so far
    std::vector<double> mean, m2;  // channel mean; sum of (x - mean)(x - mean)^T over those pixels
};

fmtc_status fmtc_fit_state_create(int C, fmtc_fit_state** out) {
    return guarded([&]() -> fmtc_status {
    if (!out) return fail(FMTC_EINVAL, "out is NULL");
    *out = nullptr;
    if (C < 1 || C > 1024) return fail(FMTC_EINVAL, "bad channel count %d", C);
    fmtc_fit_state* f = new (std::nothrow) fmtc_fit_state;
    if (!f) return fail(FMTC_ENOMEM, "host allocation failed");
    f->C = C;
    f->mean.assign(C, 0.0);
    f->m2.assign((size_t)C * C, 0.0);
    *out = f;
    return FMTC_OK;
    });
}

void fmtc_fit_state_destroy(fmtc_fit_state* state) { delete state; }

int64_t fmtc_fit_state_count(const fmtc_fit_state* state) { return state ? state->count : 0; }

fmtc_status fmtc_fit_state_update(fmtc_fit_state* state, const float* d_x, int64_t N, int C, int H, int W,
                                  fmtc_layout layout, void* hip_stream) {
    return guarded([&]() -> fmtc_status {
    if (!state || !d_x) return fail(FMTC_EINVAL, "NULL argument");
    if (!dims_ok(N, C, H, W) || state->C != C) return fail(FMTC_EINVAL, "bad dims or state has %d channels, tensor %d", state->C, C);
    if (layout != FMTC_NCHW && layout != FMTC_NHWC) return fail(FMTC_EINVAL, "bad layout");
    const int64_t HW = (int64_t)H * W, nb = N * HW;
    std::vector<double> sum, m2b;
    fmtc_status st = device_moments(d_x, N, C, HW, layout, (hipStream_t)hip_stream, &sum, &m2b);
    if (st != FMTC_OK) return st;
    // union of two pixel sets from their counts, means and centred second moments:
    // M2 = M2_a + M2_b + (n_a n_b / n) d d^T, mean = mean_a + (n_b / n) d, d = mean_b - mean_a
    const double na = (double)state->count, n = na + (double)nb;
    std::vector<double> d(C);
    for (int c = 0; c < C; c++) d[c] = sum[c] / (double)nb - state->mean[c];
    const double w = na * (double)nb / n;
    for (int i = 0; i < C; i++)
        for (int j = 0; j < C; j++) state->m2[(size_t)i * C + j] += m2b[(size_t)i * C + j] + w * d[i] * d[j];
    for (int c = 0; c < C; c++) state->mean[c] += d[c] * ((double)nb / n);
    state->count += nb;
    return FMTC_OK;
    });
}

fmtc_status fmtc_fit_state_basis(const fmtc_fit_state* state, const float* d_x, int64_t N, int C, int H, int W,
                                 fmtc_layout layout, void* hip_stream, fmtc_basis** out) {
    return guarded([&]() -> fmtc_status {
    if (!out) return fail(FMTC_EINVAL, "out is NULL");
    *out = nullptr;
    if (!state || !d_x) return fail(FMTC_EINVAL, "NULL argument");
    if (!dims_ok(N, C, H, W) || state->C != C) return fail(FMTC_EINVAL, "bad dims or state has %d channels, tensor %d", state->C, C);
    if (layout != FMTC_NCHW && layout != FMTC_NHWC) return fail(FMTC_EINVAL, "bad layout");
    if (state->count < 1) return fail(FMTC_EINVAL, "the state has seen no pixels");
    std::vector<double> cov(state->m2);
    for (size_t i = 0; i < cov.size(); i++) cov[i] /= (double)state->count;
    return finish_fit(C, state->mean, cov, d_x, N, (int64_t)H * W, layout, (hipStream_t)hip_stream, out);
    });
}

fmtc_status fmtc_basis_truncate(const fmtc_basis* basis, int keep, fmtc_basis** out) {
    return guarded([&]() -> fmtc_status {
    if (!out) return fail(FMTC_EINVAL, "out is NULL");
    *out = nullptr;
    if (!basis) return fail(FMTC_EINVAL, "basis is NULL");
    if (keep < 1 || keep > basis->C) return fail(FMTC_EINVAL, "keep must be in [1,%d], got %d", basis->C, keep);
    fmtc_basis* b = new (std::nothrow) fmtc_basis;
    if (!b) return fail(FMTC_ENOMEM, "host allocation failed");
    const int C = basis->C;
    b->C = C;
    b->Cpad = basis->Cpad;
    b->range_A = basis->range_A;
    b->T = basis->T;
    b->mu = basis->mu;
    b->eig = basis->eig;
    for (size_t i = (size_t)keep * C; i < (size_t)C * C; i++) b->T[i] = 0.f;
    fmtc_status st = upload_basis(b);
    if (st != FMTC_OK) {
        fmtc_basis_destroy(b);
        return st;
    }
    *out = b;
    return FMTC_OK;
    });
}

size_t fmtc_encode_bound(int64_t P, int C, int bits, int chunk_syms) {
    EncodePlan pl;
    if (plan_encode(P, C, bits, chunk_syms, &pl) != FMTC_OK) return 0;
    return bound_from(pl, bits);
}

size_t fmtc_workspace_size(int64_t P, int C, int bits, int chunk_syms) {
    EncodePlan pl;
    if (plan_encode(P, C, bits, chunk_syms, &pl) != FMTC_OK) return 0;
    return pl.ws.total;
}

fmtc_status fmtc_quantize(const fmtc_basis* basis, const float* d_x, int64_t N, int C, int H, int W,
                          fmtc_layout layout, int bits, uint8_t* d_syms, uint32_t* d_hist, void* d_workspace,
                          size_t ws_bytes, void* hip_stream) {
    if (!basis || !d_x || !d_syms || !d_workspace) return fail(FMTC_EINVAL, "NULL argument");
    if (!dims_ok(N, C, H, W) || basis->C != C) return fail(FMTC_EINVAL, "bad dims or basis has %d channels, tensor %d", basis->C, C);
    if (layout != FMTC_NCHW && layout != FMTC_NHWC) return fail(FMTC_EINVAL, "bad layout");
    if (bits < 2 || bits > 8) return fail(FMTC_EINVAL, "bits must be in [2,8]");
    if (!aligned(d_x, 16) || !aligned(d_syms, 16) || !aligned(d_workspace, 256)) return fail(FMTC_EINVAL, "misaligned pointer");
    EncodePlan pl;
    fmtc_status st = plan_encode(N * (int64_t)H * W, C, bits, 4096, &pl);
    if (st != FMTC_OK) return st;
    if (ws_bytes < pl.ws.off_syms) return fail(FMTC_EBUFSIZE, "workspace too small: %zu < %zu", ws_bytes, pl.ws.off_syms);
    hipStream_t s = (hipStream_t)hip_stream;
    uint8_t* w = static_cast<uint8_t*>(d_workspace);
    const CoderScratch cs = coder_scratch(w, pl);
    hipError_t e;
    int n_parts = 0;
    const float delta = fmtc_delta(basis->range_A, bits);
    if ((e = launch_project_quantize(device_view(basis), d_x, N, (int64_t)H * W, layout, delta, bits, d_syms, cs, &n_parts, s)) != hipSuccess)
        return hip_fail(e, "project/quantize kernel");
    if (d_hist && (e = launch_histogram_sum(cs.hist_parts, n_parts, bits, d_hist, s)) != hipSuccess)
        return hip_fail(e, "histogram reduction");
    return FMTC_OK;
}

fmtc_status fmtc_encode(const fmtc_basis* basis, const float* d_x, int64_t N, int C, int H, int W,
                        fmtc_layout layout, int bits, int chunk_syms, void* d_stream_out, size_t cap,
                        uint64_t* d_out_bytes, void* d_workspace, size_t ws_bytes, void* hip_stream) {
    if (!basis || !d_x || !d_stream_out || !d_workspace) return fail(FMTC_EINVAL, "NULL argument");
    if (!dims_ok(N, C, H, W) || basis->C != C) return fail(FMTC_EINVAL, "bad dims or basis has %d channels, tensor %d", basis->C, C);
    if (layout != FMTC_NCHW && layout != FMTC_NHWC) return fail(FMTC_EINVAL, "bad layout");
    if (!aligned(d_x, 16) || !aligned(d_stream_out, 16) || !aligned(d_workspace, 256) || !aligned(d_out_bytes, 8))
        return fail(FMTC_EINVAL, "misaligned pointer");
    EncodePlan pl;
    const int64_t HW = (int64_t)H * W;
    fmtc_status st = plan_encode(N * HW, C, bits, chunk_syms, &pl);
    if (st != FMTC_OK) return st;
    if (ws_bytes < pl.ws.total) return fail(FMTC_EBUFSIZE, "workspace too small: %zu < %zu", ws_bytes, pl.ws.total);
    if (cap < bound_from(pl, bits)) return fail(FMTC_EBUFSIZE, "stream capacity too small: %zu < %zu", cap, bound_from(pl, bits));
    hipStream_t s = (hipStream_t)hip_stream;
    uint8_t* w = static_cast<uint8_t*>(d_workspace);
    const CoderScratch cs = coder_scratch(w, pl);
    uint8_t* syms = w + pl.ws.off_syms;
    hipError_t e;
    int n_parts = 0;
    const float delta = fmtc_delta(basis->range_A, bits);
    if ((e = launch_project_quantize(device_view(basis), d_x, N, HW, layout, delta, bits, syms, cs, &n_parts, s)) != hipSuccess)
        return hip_fail(e, "project/quantize kernel");
    return run_coder(syms, pl, cs, n_parts, bits, delta, w, static_cast<uint8_t*>(d_stream_out), cap, d_out_bytes, s);
}

// ---- code table fixed at calibration time ----
static bool lengths_complete(const uint8_t* len, int bits, uint32_t* max_len) {
    // Kraft sum of a complete prefix code: sum 2^-len == 1, in units of 2^-48
    unsigned long long sum = 0;
    uint32_t mx = 0;
    for (int s = 0; s < (1 << bits); s++) {
        if (len[s] < 1 || len[s] > kMaxLen) return false;
        sum += 1ull << (kMaxLen - len[s]);
        if (len[s] > mx) mx = len[s];
    }
    *max_len = mx;
    return sum == (1ull << kMaxLen);
}

// The decoder's tables for the handle's code lengths (t->lengths), on the given stream; synchronises it.
static fmtc_status make_decode_tables(fmtc_table* t, hipStream_t s) {
    uint8_t* d_len = nullptr;
    uint32_t* d_ok = nullptr;
    uint32_t ok = 0;
    hipError_t e;
    if ((e = hipMalloc(&t->d_dec_tables, prebuilt_decode_tables_bytes())) != hipSuccess ||
        (e = hipMalloc((void**)&d_len, 256)) != hipSuccess || (e = hipMalloc((void**)&d_ok, 4)) != hipSuccess) {
        if (d_len) (void)hipFree(d_len);
        return fail(FMTC_ENOMEM, "hipMalloc decode tables: %s", hipGetErrorString(e));
    }
    if ((e = hipMemcpyAsync(d_len, t->lengths, 256, hipMemcpyHostToDevice, s)) == hipSuccess &&
        (e = launch_build_decode_tables(d_len, t->bits, t->d_dec_tables, d_ok, s)) == hipSuccess &&
        (e = hipMemcpyAsync(&ok, d_ok, 4, hipMemcpyDeviceToHost, s)) == hipSuccess)
        e = hipStreamSynchronize(s);
    (void)hipFree(d_len);
    (void)hipFree(d_ok);
    if (e != hipSuccess) return hip_fail(e, "decode table build");
    if (!ok) return fail(FMTC_EHIP, "decode tables rejected the code lengths");
    return FMTC_OK;
}

void fmtc_table_destroy(fmtc_table* t) {
    if (!t) return;
    if (t->d_enc_table) (void)hipFree(t->d_enc_table);
    if (t->d_dec_tables) (void)hipFree(t->d_dec_tables);
    delete t;
}

fmtc_status fmtc_table_import(const uint8_t* h_lengths, int bits, fmtc_table** out) {
    return guarded([&]() -> fmtc_status {
    if (!h_lengths || !out) return fail(FMTC_EINVAL, "NULL argument");
    if (bits < 2 || bits > 8) return fail(FMTC_EINVAL, "bits must be in [2,8]");
    uint32_t max_len = 0;
    if (!lengths_complete(h_lengths, bits, &max_len))
        return fail(FMTC_EINVAL, "lengths are not those of a complete prefix code over %d symbols", 1 << bits);
    fmtc_table* t = new (std::nothrow) fmtc_table;
    if (!t) return fail(FMTC_ENOMEM, "host allocation failed");
    t->bits = bits;
    t->max_len = max_len;
    memcpy(t->lengths, h_lengths, (size_t)1 << bits);
    hipError_t e;
    uint8_t* d_len = nullptr;
    if ((e = hipGetDevice(&t->device)) != hipSuccess || (e = hipMalloc((void**)&t->d_enc_table, 256 * sizeof(uint64_t))) != hipSuccess ||
        (e = hipMalloc((void**)&d_len, 256)) != hipSuccess) {
        fmtc_table_destroy(t);
        return fail(FMTC_ENOMEM, "hipMalloc table: %s", hipGetErrorString(e));
    }
    if ((e = hipMemcpy(d_len, t->lengths, 256, hipMemcpyHostToDevice)) == hipSuccess &&
        (e = launch_table_from_lengths(d_len, bits, t->d_enc_table, nullptr)) == hipSuccess)
        e = hipStreamSynchronize(nullptr);
    (void)hipFree(d_len);
    if (e != hipSuccess) {
        fmtc_table_destroy(t);
        return hip_fail(e, "table upload");
    }
    const fmtc_status st = make_decode_tables(t, nullptr);
    if (st != FMTC_OK) {
        fmtc_table_destroy(t);
        return st;
    }
    *out = t;
    return FMTC_OK;
    });
}

fmtc_status fmtc_table_export(const fmtc_table* t, uint8_t* h_lengths, int* bits) {
    if (!t) return fail(FMTC_EINVAL, "NULL argument");
    if (h_lengths) memcpy(h_lengths, t->lengths, 256);
    if (bits) *bits = t->bits;
    return FMTC_OK;
}

fmtc_status fmtc_fit_table(const fmtc_basis* basis, const float* d_x, int64_t N, int C, int H, int W,
                           fmtc_layout layout, int bits, void* hip_stream, fmtc_table** out) {
    return guarded([&]() -> fmtc_status {
    if (!basis || !d_x || !out) return fail(FMTC_EINVAL, "NULL argument");
    if (!dims_ok(N, C, H, W) || basis->C != C) return fail(FMTC_EINVAL, "bad dims or basis has %d channels, tensor %d", basis->C, C);
    if (layout != FMTC_NCHW && layout != FMTC_NHWC) return fail(FMTC_EINVAL, "bad layout");
    if (bits < 2 || bits > 8) return fail(FMTC_EINVAL, "bits must be in [2,8]");
    if (!aligned(d_x, 16)) return fail(FMTC_EINVAL, "misaligned pointer");
    EncodePlan pl;
    const int64_t HW = (int64_t)H * W;
    fmtc_status st = plan_encode(N * HW, C, bits, 4096, &pl);
    if (st != FMTC_OK) return st;
    hipStream_t s = (hipStream_t)hip_stream;
    fmtc_table* t = new (std::nothrow) fmtc_table;
    if (!t) return fail(FMTC_ENOMEM, "host allocation failed");
    t->bits = bits;
    uint8_t *ws = nullptr, *d_len = nullptr;
    hipError_t e;
    if ((e = hipGetDevice(&t->device)) != hipSuccess || (e = hipMalloc((void**)&t->d_enc_table, 256 * sizeof(uint64_t))) != hipSuccess ||
        (e = hipMalloc((void**)&ws, pl.ws.total)) != hipSuccess || (e = hipMalloc((void**)&d_len, 256)) != hipSuccess) {
        if (ws) (void)hipFree(ws);
        fmtc_table_destroy(t);
        return fail(FMTC_ENOMEM, "hipMalloc table fit: %s", hipGetErrorString(e));
    }
    const CoderScratch cs = coder_scratch(ws, pl);
    int n_parts = 0;
    const float delta = fmtc_delta(basis->range_A, bits);
    if ((e = launch_project_quantize(device_view(basis), d_x, N, HW, layout, delta, bits, ws + pl.ws.off_syms, cs, &n_parts, s)) == hipSuccess &&
        (e = launch_table_from_hist(cs.hist_parts, n_parts, bits, 1u, t->d_enc_table, d_len, s)) == hipSuccess &&
        (e = hipMemcpyAsync(t->lengths, d_len, 256, hipMemcpyDeviceToHost, s)) == hipSuccess)
        e = hipStreamSynchronize(s);
    (void)hipFree(ws);
    (void)hipFree(d_len);
    if (e != hipSuccess) {
        fmtc_table_destroy(t);
        return hip_fail(e, "table fit");
    }
    if (!lengths_complete(t->lengths, bits, &t->max_len)) {
        fmtc_table_destroy(t);
        return fail(FMTC_EHIP, "table fit produced an incomplete code");
    }
    st = make_decode_tables(t, s);
    if (st != FMTC_OK) {
        fmtc_table_destroy(t);
        return st;
    }
    *out = t;
    return FMTC_OK;
    });
}

static size_t static_bound_from(const EncodePlan& pl, uint32_t max_len) {
    // every chunk: its symbols at the longest code, rounded up to whole words
    const uint64_t full = (uint64_t)pl.g.chunk_syms * max_len;
    return pl.g.off_payload + 4 * (size_t)(((full + 31) / 32) * pl.g.n_chunks);
}

size_t fmtc_encode_static_bound(const fmtc_table* t, int64_t P, int C, int chunk_syms) {
    EncodePlan pl;
    if (!t || plan_encode(P, C, t->bits, chunk_syms, &pl) != FMTC_OK) return 0;
    return static_bound_from(pl, t->max_len);
}

fmtc_status fmtc_encode_static(const fmtc_basis* basis, const fmtc_table* t, const float* d_x, int64_t N, int C, int H,
                               int W, fmtc_layout layout, int chunk_syms, void* d_stream_out, size_t cap,
                               uint64_t* d_out_bytes, void* d_workspace, size_t ws_bytes, void* hip_stream) {
    if (!basis || !t || !d_x || !d_stream_out || !d_workspace) return fail(FMTC_EINVAL, "NULL argument");
    if (!dims_ok(N, C, H, W) || basis->C != C) return fail(FMTC_EINVAL, "bad dims or basis has %d channels, tensor %d", basis->C, C);
    if (layout != FMTC_NCHW && layout != FMTC_NHWC) return fail(FMTC_EINVAL, "bad layout");
    if (!aligned(d_x, 16) || !aligned(d_stream_out, 16) || !aligned(d_workspace, 256) || !aligned(d_out_bytes, 8))
        return fail(FMTC_EINVAL, "misaligned pointer");
    const int bits = t->bits;
    EncodePlan pl;
    const int64_t HW = (int64_t)H * W;
    fmtc_status st = plan_encode(N * HW, C, bits, chunk_syms, &pl);
    if (st != FMTC_OK) return st;
    if (ws_bytes < pl.ws.total) return fail(FMTC_EBUFSIZE, "workspace too small: %zu < %zu", ws_bytes, pl.ws.total);
    if (cap < pl.g.off_payload) return fail(FMTC_EBUFSIZE, "stream capacity too small: %zu < %zu", cap, (size_t)pl.g.off_payload);
    hipStream_t s = (hipStream_t)hip_stream;
    uint8_t* w = static_cast<uint8_t*>(d_workspace);
    const CoderScratch cs = coder_scratch(w, pl);
    uint8_t* syms = w + pl.ws.off_syms;
    const float delta = fmtc_delta(basis->range_A, bits);
    const uint64_t cap_words = (cap - pl.g.off_payload) / 4;
    hipError_t e;
    int n_parts = 0;
    // one kernel where the shape allows it: the coder's counters are cleared first, since the kernel that counts
    // in them is also the one that would clear them
    {
        PackParams pk = pack_params(nullptr, pl.g, bits, delta, cs, 0, t->d_enc_table, static_cast<uint8_t*>(d_stream_out),
                                    cap_words, d_out_bytes);
        pk.static_max_len = t->max_len;
        if (!test_option(kTestStaticTwoKernels) && encode_static_fused_applies(C, layout, (uint32_t)chunk_syms, cs.n_groups)) {
            static_assert(sizeof(CoderCtrl) % 4 == 0, "control block is cleared as words");
            const size_t clear_bytes = pl.ws.off_lookback + sizeof(uint64_t) * (size_t)cs.n_groups - pl.ws.off_ctrl;
            if ((e = launch_fill_zero(reinterpret_cast<uint32_t*>(w + pl.ws.off_ctrl), clear_bytes / 4, s)) != hipSuccess)
                return hip_fail(e, "clear kernel");
            e = launch_encode_static_fused(device_view(basis), d_x, N, HW, layout, delta, bits, cs, pk, s);
            if (e == hipSuccess) return FMTC_OK;
            if (e != hipErrorNotSupported) return hip_fail(e, "fused encode kernel");
        }
    }
    if ((e = launch_project_quantize(device_view(basis), d_x, N, HW, layout, delta, bits, syms, cs, &n_parts, s)) != hipSuccess)
        return hip_fail(e, "project/quantize kernel");
    if ((e = launch_coder_static(syms, pl.g, bits, delta, cs, t->d_enc_table, t->max_len, static_cast<uint8_t*>(d_stream_out),
                                 cap_words, d_out_bytes, s)) != hipSuccess)
        return hip_fail(e, "coder kernel");
    return FMTC_OK;
}

fmtc_status fmtc_code_symbols(const uint8_t* d_syms, int64_t P, int C, int bits, int chunk_syms, float delta,
                              void* d_stream_out, size_t cap, uint64_t* d_out_bytes, void* d_workspace,
                              size_t ws_bytes, void* hip_stream) {
    if (!d_syms || !d_stream_out || !d_workspace) return fail(FMTC_EINVAL, "NULL argument");
    if (!(delta > 0.f)) return fail(FMTC_EINVAL, "delta must be > 0");
    if (!aligned(d_syms, 16) || !aligned(d_stream_out, 16) || !aligned(d_workspace, 256) || !aligned(d_out_bytes, 8))
        return fail(FMTC_EINVAL, "misaligned pointer");
    EncodePlan pl;
    fmtc_status st = plan_encode(P, C, bits, chunk_syms, &pl);
    if (st != FMTC_OK) return st;
    if (ws_bytes < pl.ws.off_syms) return fail(FMTC_EBUFSIZE, "workspace too small: %zu < %zu", ws_bytes, pl.ws.off_syms);
    if (cap < bound_from(pl, bits)) return fail(FMTC_EBUFSIZE, "stream capacity too small: %zu < %zu", cap, bound_from(pl, bits));
    hipStream_t s = (hipStream_t)hip_stream;
    uint8_t* w = static_cast<uint8_t*>(d_workspace);
    const CoderScratch cs = coder_scratch(w, pl);
    hipError_t e;
    int n_parts = 0;
    if ((e = launch_histogram(d_syms, pl.V, bits, cs, &n_parts, s)) != hipSuccess) return hip_fail(e, "histogram kernel");
    return run_coder(d_syms, pl, cs, n_parts, bits, delta, w, static_cast<uint8_t*>(d_stream_out), cap, d_out_bytes, s);
}

static fmtc_status decode_common(const fmtc_basis* basis, const void* d_stream_in, size_t bytes, int64_t P, int C,
                                 int64_t HW, int layout, int bits, float* d_xhat, uint8_t* d_syms,
                                 uint32_t* d_err_flag, void* hip_stream, const void* d_prebuilt = nullptr) {
    if (!d_stream_in || !d_err_flag) return fail(FMTC_EINVAL, "NULL argument");
    if (bits < 2 || bits > 8) return fail(FMTC_EINVAL, "bits must be in [2,8]");
    if (!aligned(d_stream_in, 16) || !aligned(d_err_flag, 4) || !aligned(d_xhat, 16) || !aligned(d_syms, 16))
        return fail(FMTC_EINVAL, "misaligned pointer");
    Geometry g;
    if (!make_geometry(P, C, 4096, &g)) return fail(FMTC_EINVAL, "bad geometry");
    if ((long double)P * C >= 4294967296.0L) return fail(FMTC_EINVAL, "tensor too large: V must be < 2^32");
    hipStream_t s = (hipStream_t)hip_stream;
    hipError_t e;
    BasisDevice view;
    if (basis) view = device_view(basis);
    if ((e = launch_decode(basis ? &view : nullptr, static_cast<const uint8_t*>(d_stream_in), bytes, g, bits, HW,
                           layout, d_xhat, d_syms, d_err_flag, d_prebuilt, s)) != hipSuccess)
        return hip_fail(e, "decode kernel");
    return FMTC_OK;
}

fmtc_status fmtc_decode(const fmtc_basis* basis, const void* d_stream_in, size_t bytes, float* d_xhat, int64_t N,
                        int C, int H, int W, fmtc_layout layout, int bits, uint32_t* d_err_flag, void* hip_stream) {
    if (!basis || !d_xhat) return fail(FMTC_EINVAL, "NULL argument");
    if (!dims_ok(N, C, H, W) || basis->C != C) return fail(FMTC_EINVAL, "bad dims or basis has %d channels, tensor %d", basis->C, C);
    if (layout != FMTC_NCHW && layout != FMTC_NHWC) return fail(FMTC_EINVAL, "bad layout");
    const int64_t HW = (int64_t)H * W;
    return decode_common(basis, d_stream_in, bytes, N * HW, C, HW, layout, bits, d_xhat, nullptr, d_err_flag, hip_stream);
}

fmtc_status fmtc_decode_static(const fmtc_basis* basis, const fmtc_table* table, const void* d_stream_in, size_t bytes,
                               float* d_xhat, int64_t N, int C, int H, int W, fmtc_layout layout,
                               uint32_t* d_err_flag, void* hip_stream) {
    if (!basis || !table || !d_xhat) return fail(FMTC_EINVAL, "NULL argument");
    if (!dims_ok(N, C, H, W) || basis->C != C) return fail(FMTC_EINVAL, "bad dims or basis has %d channels, tensor %d", basis->C, C);
    if (layout != FMTC_NCHW && layout != FMTC_NHWC) return fail(FMTC_EINVAL, "bad layout");
    const int64_t HW = (int64_t)H * W;
    return decode_common(basis, d_stream_in, bytes, N * HW, C, HW, layout, table->bits, d_xhat, nullptr, d_err_flag,
                         hip_stream, table->d_dec_tables);
}

fmtc_status fmtc_decode_symbols(const void* d_stream_in, size_t bytes, int64_t P, int C, int bits, uint8_t* d_syms,
                                uint32_t* d_err_flag, void* hip_stream) {
    if (!d_syms) return fail(FMTC_EINVAL, "NULL argument");
    if (P < 1 || C < 1 || C > 1024) return fail(FMTC_EINVAL, "bad dims");
    return decode_common(nullptr, d_stream_in, bytes, P, C, 1, FMTC_NHWC, bits, nullptr, d_syms, d_err_flag, hip_stream);
}

fmtc_status fmtc_stream_info(const void* h_header, size_t header_bytes, int* bits, int* C, int64_t* P,
                             int* px_per_chunk, int64_t* n_chunks, float* delta, uint64_t* payload_bits,
                             uint64_t* stream_bytes) {
    if (!h_header || header_bytes < (size_t)kHeaderBytes) return fail(FMTC_EINVAL, "need the 64 header bytes");
    Header h;
    memcpy(&h, h_header, sizeof h);
    if (h.magic != kMagic || h.version != 1) return fail(FMTC_ECORRUPT, "not a stream header");
    if (h.bits < 2 || h.bits > 8 || h.C < 1 || h.C > 1024 || h.px_per_chunk < 1 || h.P < 1)
        return fail(FMTC_ECORRUPT, "header fields out of range");
    const uint64_t nch = (h.P + h.px_per_chunk - 1) / h.px_per_chunk;
    const uint64_t spc = ((uint64_t)h.px_per_chunk * h.C + kSubSyms - 1) / kSubSyms;
    if (nch != h.n_chunks || spc != h.subs_per_chunk) return fail(FMTC_ECORRUPT, "header geometry inconsistent");
    const size_t off_sub = align_up(kHeaderBytes + kLenTableBytes + 4 * ((size_t)nch + 1), 16);
    const size_t off_pay = align_up(off_sub + 2 * (size_t)nch * spc, 16);
    if (bits) *bits = h.bits;
    if (C) *C = (int)h.C;
    if (P) *P = (int64_t)h.P;
    if (px_per_chunk) *px_per_chunk = (int)h.px_per_chunk;
    if (n_chunks) *n_chunks = (int64_t)nch;
    if (delta) *delta = h.delta;
    if (payload_bits) *payload_bits = h.payload_bits;
    if (stream_bytes) *stream_bytes = off_pay + 4 * h.payload_words;
    return FMTC_OK;
}


fmtc_status fmtc_basis8_create(const fmtc_basis* basis, float act_scale, fmtc_basis8** out) {
    return guarded([&]() -> fmtc_status {
    if (!out) return fail(FMTC_EINVAL, "out is NULL");
    *out = nullptr;
    if (!basis) return fail(FMTC_EINVAL, "basis is NULL");
    if (!(act_scale > 0.f) || !std::isfinite(act_scale)) return fail(FMTC_EINVAL, "act_scale must be a positive number");
    fmtc_basis8* b = new (std::nothrow) fmtc_basis8;
    if (!b) return fail(FMTC_ENOMEM, "host allocation failed");
    const int C = basis->C;
    b->C = C;
    b->act_scale = act_scale;
    b->range_A = basis->range_A;
    double amax = 0.0;
    for (float v : basis->T) amax = std::fabs((double)v) > amax ? std::fabs((double)v) : amax;
    b->scale_T = (float)(amax / 127.0);
    if (!(b->scale_T > 0.f)) b->scale_T = 1.f;
    b->Tq.resize((size_t)C * C);
    for (size_t i = 0; i < b->Tq.size(); i++) {
        double r = std::nearbyint((double)basis->T[i] / (double)b->scale_T);
        r = r > 127.0 ? 127.0 : (r < -127.0 ? -127.0 : r);
        b->Tq[i] = (int8_t)(int)r;
    }
    b->mean_fix.resize(C);
    for (int c = 0; c < C; c++) {
        const double m = std::nearbyint((double)basis->mu[c] / (double)act_scale * 256.0);
        if (!(std::fabs(m) < 1073741824.0)) {
            delete b;
            return fail(FMTC_EINVAL, "mean of channel %d is out of range for this activation scale", c);
        }
        b->mean_fix[c] = (int32_t)m;
    }
    fmtc_status st = upload_basis8(b);
    if (st != FMTC_OK) {
        fmtc_basis8_destroy(b);
        return st;
    }
    *out = b;
    return FMTC_OK;
    });
}

void fmtc_basis8_destroy(fmtc_basis8* b) {
    if (!b) return;
    if (b->d_block) (void)hipFree(b->d_block);
    delete b;
}

fmtc_status fmtc_basis8_export(const fmtc_basis8* b, int8_t* h_Tq, float* scale_T, int32_t* h_mean_fix,
                               float* act_scale, float* range_A) {
    if (!b) return fail(FMTC_EINVAL, "basis is NULL");
    if (h_Tq) memcpy(h_Tq, b->Tq.data(), b->Tq.size());
    if (scale_T) *scale_T = b->scale_T;
    if (h_mean_fix) memcpy(h_mean_fix, b->mean_fix.data(), sizeof(int32_t) * b->mean_fix.size());
    if (act_scale) *act_scale = b->act_scale;
    if (range_A) *range_A = b->range_A;
    return FMTC_OK;
}

static fmtc_status check_u8_call(const fmtc_basis8* b, const void* a, const void* c, int64_t N, int C, int H, int W,
                                 fmtc_layout layout, int bits) {
    if (!b || !a || !c) return fail(FMTC_EINVAL, "NULL argument");
    if (!dims_ok(N, C, H, W) || b->C != C) return fail(FMTC_EINVAL, "bad dims or basis has %d channels, tensor %d", b->C, C);
    if (layout != FMTC_NCHW && layout != FMTC_NHWC) return fail(FMTC_EINVAL, "bad layout");
    if (bits < 2 || bits > 8) return fail(FMTC_EINVAL, "bits must be in [2,8]");
    if (!aligned(a, 16) || !aligned(c, 16)) return fail(FMTC_EINVAL, "misaligned pointer");
    return FMTC_OK;
}

fmtc_status fmtc_quantize_u8(const fmtc_basis8* basis, const uint8_t* d_xq, int64_t N, int C, int H, int W,
                             fmtc_layout layout, int bits, uint8_t* d_syms, void* hip_stream) {
    fmtc_status st = check_u8_call(basis, d_xq, d_syms, N, C, H, W, layout, bits);
    if (st != FMTC_OK) return st;
    const int64_t HW = (int64_t)H * W;
    const double delta = (double)fmtc_delta(basis->range_A, bits);
    const double g = ((double)basis->scale_T * (double)basis->act_scale) / (256.0 * delta);
    hipError_t e = launch_quantize_u8(basis->view, d_xq, N * HW, HW, layout, bits, g, d_syms, nullptr, nullptr,
                                      (hipStream_t)hip_stream);
    if (e != hipSuccess) return hip_fail(e, "8-bit projection kernel");
    return FMTC_OK;
}

fmtc_status fmtc_reconstruct_u8(const fmtc_basis8* basis, const uint8_t* d_syms, int64_t N, int C, int H, int W,
                                fmtc_layout layout, int bits, uint8_t* d_xq_hat, void* hip_stream) {
    fmtc_status st = check_u8_call(basis, d_syms, d_xq_hat, N, C, H, W, layout, bits);
    if (st != FMTC_OK) return st;
    const int64_t HW = (int64_t)H * W;
    const double delta = (double)fmtc_delta(basis->range_A, bits);
    const double h = ((double)basis->scale_T * delta * 256.0) / (double)basis->act_scale;  // the kernel gets h / 256 (exact)
    hipError_t e = launch_reconstruct_u8(basis->view, d_syms, N * HW, HW, layout, bits, h / 256.0, d_xq_hat, (hipStream_t)hip_stream);
    if (e != hipSuccess) return hip_fail(e, "8-bit reconstruction kernel");
    return FMTC_OK;
}

fmtc_status fmtc_encode_u8(const fmtc_basis8* basis, const uint8_t* d_xq, int64_t N, int C, int H, int W,
                           fmtc_layout layout, int bits, int chunk_syms, void* d_stream_out, size_t cap,
                           uint64_t* d_out_bytes, void* d_workspace, size_t ws_bytes, void* hip_stream) {
    if (!d_stream_out || !d_workspace) return fail(FMTC_EINVAL, "NULL argument");
    fmtc_status st = check_u8_call(basis, d_xq, d_stream_out, N, C, H, W, layout, bits);
    if (st != FMTC_OK) return st;
    if (!aligned(d_workspace, 256) || !aligned(d_out_bytes, 8)) return fail(FMTC_EINVAL, "misaligned pointer");
    EncodePlan pl;
    const int64_t P = N * (int64_t)H * W;
    st = plan_encode(P, C, bits, chunk_syms, &pl);
    if (st != FMTC_OK) return st;
    if (ws_bytes < pl.ws.total) return fail(FMTC_EBUFSIZE, "workspace too small: %zu < %zu", ws_bytes, pl.ws.total);
    if (cap < bound_from(pl, bits)) return fail(FMTC_EBUFSIZE, "stream capacity too small: %zu < %zu", cap, bound_from(pl, bits));
    uint8_t* w = static_cast<uint8_t*>(d_workspace);
    uint8_t* syms = w + pl.ws.off_syms;
    const CoderScratch cs = coder_scratch(w, pl);
    const float delta = fmtc_delta(basis->range_A, bits);
    const double g = ((double)basis->scale_T * (double)basis->act_scale) / (256.0 * (double)delta);
    hipStream_t s = (hipStream_t)hip_stream;
    int n_parts = 0;
    hipError_t e = launch_quantize_u8(basis->view, d_xq, P, (int64_t)H * W, layout, bits, g, syms, &cs, &n_parts, s);
    if (e != hipSuccess) return hip_fail(e, "8-bit projection kernel");
    return run_coder(syms, pl, cs, n_parts, bits, delta, w, static_cast<uint8_t*>(d_stream_out), cap, d_out_bytes, s);
}

fmtc_status fmtc_decode_u8(const fmtc_basis8* basis, const void* d_stream_in, size_t bytes, uint8_t* d_xq_hat,
                           int64_t N, int C, int H, int W, fmtc_layout layout, int bits, uint32_t* d_err_flag,
                           void* d_workspace, size_t ws_bytes, void* hip_stream) {
    if (!d_stream_in || !d_err_flag) return fail(FMTC_EINVAL, "NULL argument");
    fmtc_status st = check_u8_call(basis, d_stream_in, d_xq_hat, N, C, H, W, layout, bits);
    if (st != FMTC_OK) return st;
    const int64_t P = N * (int64_t)H * W;
    if (!aligned(d_err_flag, 4)) return fail(FMTC_EINVAL, "misaligned pointer");
    if (C > 128) {  // wider tensors go through the symbols in the workspace
        if (!d_workspace || !aligned(d_workspace, 16)) return fail(FMTC_EINVAL, "workspace is NULL or misaligned");
        if (ws_bytes < (size_t)P * (size_t)C) return fail(FMTC_EBUFSIZE, "workspace too small: %zu < %zu", ws_bytes, (size_t)P * (size_t)C);
    }
    {   // up to 128 channels: one kernel, the symbols never leave the chip
        Geometry g;
        if (!make_geometry(P, C, 4096, &g)) return fail(FMTC_EINVAL, "bad geometry");
        const double delta = (double)fmtc_delta(basis->range_A, bits);
        const double h = ((double)basis->scale_T * delta * 256.0) / (double)basis->act_scale;
        bool applies = false;
        hipError_t e = launch_decode_u8(basis->view, static_cast<const uint8_t*>(d_stream_in), bytes, g, bits,
                                        (int64_t)H * W, layout, h / 256.0, d_xq_hat, d_err_flag, &applies, (hipStream_t)hip_stream);
        if (e != hipSuccess) return hip_fail(e, "8-bit decode kernel");
        if (applies) return FMTC_OK;
    }
    uint8_t* syms = static_cast<uint8_t*>(d_workspace);
    st = fmtc_decode_symbols(d_stream_in, bytes, P, C, bits, syms, d_err_flag, hip_stream);
    if (st != FMTC_OK) return st;
    return fmtc_reconstruct_u8(basis, syms, N, C, H, W, layout, bits, d_xq_hat, hip_stream);
}

// The same encoder with the workspace in the library's own device array (see `scratch` above): no allocation here
// or below (the launch sequence of fmtc_encode makes none), so the call fits callers that may not allocate.
fmtc_status fmtc_encode_noalloc(const fmtc_basis* basis, const float* d_x, int64_t N, int C, int H, int W,
                                fmtc_layout layout, int bits, int chunk_syms, void* d_stream_out, size_t cap,
                                uint64_t* d_out_bytes, void* hip_stream) {
    if (!dims_ok(N, C, H, W)) return fail(FMTC_EINVAL, "bad dims");
    EncodePlan pl;
    fmtc_status st = plan_encode(N * (int64_t)H * W, C, bits, chunk_syms, &pl);
    if (st != FMTC_OK) return st;
    if (pl.ws.total > kNoAllocScratchBytes)
        return fail(FMTC_EBUFSIZE, "tensor too large for fmtc_encode_noalloc: it needs %zu bytes of scratch, the "
                    "library's array holds %zu (use fmtc_encode with a workspace)", pl.ws.total, kNoAllocScratchBytes);
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= kNoAllocMaxDevices) return fail(FMTC_EINVAL, "device index %d not supported", dev);
    uint8_t* ptr = g_noalloc_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {  // first call on this device: this GPU's copy of the array (every thread gets the same answer)
        void* sym = nullptr;
        if ((e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch))) != hipSuccess) return hip_fail(e, "hipGetSymbolAddress");
        if (!sym || !aligned(sym, 256)) return fail(FMTC_EHIP, "scratch array not resolved");
        ptr = static_cast<uint8_t*>(sym);
        g_noalloc_scratch_ptr[dev].store(ptr, std::memory_order_release);
    }
    return fmtc_encode(basis, d_x, N, C, H, W, layout, bits, chunk_syms, d_stream_out, cap, d_out_bytes, ptr,
                       kNoAllocScratchBytes, hip_stream);
}

}  // extern "C"
