/*
 * fmtc_oracle.c -- plain, slow, fp64 CPU oracle for feature-map transform coding.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the reference the GPU library is
 * checked against.  It shares no code, header, table or helper with the GPU
 * library, and nothing in the product path may call it.  Only tests, the
 * smoke check and the benchmark's cpu_baseline leg link it.
 *
 * The method (paper section 3 and section 3.1):
 *   encode:  y = T (x - mu)            affine decorrelating transform per 1x1xC block
 *            q = Q_Delta(y)            uniform scalar quantizer, one step for all channels
 *            VLC                       Huffman code over the quantizer output
 *   decode:  VLD, inverse quantizer (levels scaled back), inverse transform T^T
 * T is the PCA / KLT basis of the channel covariance fitted on a calibration
 * batch (section 3, section 3.1 "Linear transform").
 *
 * All arithmetic is fp64 on fp32 inputs.  T, mu, the range A and the step
 * Delta are rounded to fp32 once; every later step consumes those fp32 values.
 * No blocking, fusion or reordering: each function is one step of the method.
 *
 * Beyond that: the table fixed at calibration time (counts + 1), the
 * truncated projection and reconstruction (section 4 "Ablation study"), the
 * dynamic range measured on a given tensor (calibration over several
 * tensors), and the integer arithmetic of the 8-bit basis with 8-bit
 * activations (section 3.1 "Linear transform", section 5), which is exact
 * integers plus one correctly rounded fp64 operation per value.
 *
 * Pinned by tests/test_oracle_*.py (closed forms, hand-worked codes, Kraft
 * equality, brute-force optimality, entropy bounds, numpy.linalg.eigh
 * cross-check; truncation: the dropped eigenvalues' sum and a two-channel hand
 * case; 8-bit path: hand cases with ties and clamps, a brute force in exact
 * rationals, the floating-point functions above on the dequantized inputs).
 * Parity unpinned: none of the functions below; the absolute
 * bits/value of the paper's tables (real networks) cannot be reproduced here.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK 0
#define ORC_EINVAL 1
#define ORC_EBUFSIZE 2
#define ORC_ECORRUPT 3
#define ORC_ENOMEM 4

#define LAYOUT_NCHW 0
#define LAYOUT_NHWC 1

#define MAX_SYMS 256
#define MAX_LEN 48
#define SUB_SYMS 64
#define HEADER_BYTES 64
#define LEN_TABLE_BYTES 256

/* element (n, c, hw) of a tensor with logical dims (N, C, H*W) */
static size_t x_index(int layout, int64_t n, int c, int64_t hw, int C, int64_t HW)
{
    if (layout == LAYOUT_NHWC) return ((size_t)n * (size_t)HW + (size_t)hw) * (size_t)C + (size_t)c;
    return ((size_t)n * (size_t)C + (size_t)c) * (size_t)HW + (size_t)hw;
}

/* ------------------------------------------------------------------ fit */

/* Symmetric eigendecomposition by cyclic Jacobi rotations (fp64).
 * a: n*n symmetric, destroyed (diagonal -> eigenvalues); v: n*n, columns -> eigenvectors. */
static void jacobi_eigh(double *a, double *v, int n)
{
    for (int i = 0; i < n; i++)
        for (int j = 0; j < n; j++) v[(size_t)i * n + j] = (i == j) ? 1.0 : 0.0;
    double fro = 0.0;
    for (size_t i = 0; i < (size_t)n * n; i++) fro += a[i] * a[i];
    fro = sqrt(fro);
    if (fro == 0.0) return;
    for (int sweep = 0; sweep < 100; sweep++) {
        double off = 0.0;
        for (int p = 0; p < n; p++)
            for (int q = p + 1; q < n; q++) off += 2.0 * a[(size_t)p * n + q] * a[(size_t)p * n + q];
        if (sqrt(off) <= 1e-14 * fro) break;
        for (int p = 0; p < n; p++) {
            for (int q = p + 1; q < n; q++) {
                double apq = a[(size_t)p * n + q];
                if (apq == 0.0) continue;
                double app = a[(size_t)p * n + p], aqq = a[(size_t)q * n + q];
                double theta = (aqq - app) / (2.0 * apq);
                double t = (theta >= 0.0 ? 1.0 : -1.0) / (fabs(theta) + sqrt(theta * theta + 1.0));
                double c = 1.0 / sqrt(t * t + 1.0), s = t * c;
                /* A <- J^T A J with J the rotation in the (p,q) plane */
                for (int k = 0; k < n; k++) {
                    double akp = a[(size_t)k * n + p], akq = a[(size_t)k * n + q];
                    a[(size_t)k * n + p] = c * akp - s * akq;
                    a[(size_t)k * n + q] = s * akp + c * akq;
                }
                for (int k = 0; k < n; k++) {
                    double apk = a[(size_t)p * n + k], aqk = a[(size_t)q * n + k];
                    a[(size_t)p * n + k] = c * apk - s * aqk;
                    a[(size_t)q * n + k] = s * apk + c * aqk;
                }
                for (int k = 0; k < n; k++) {
                    double vkp = v[(size_t)k * n + p], vkq = v[(size_t)k * n + q];
                    v[(size_t)k * n + p] = c * vkp - s * vkq;
                    v[(size_t)k * n + q] = s * vkp + c * vkq;
                }
            }
        }
    }
}

/* Channel mean and covariance (normalised by 1/P) of a calibration tensor
 * (section 3: x ~ N(mu, Sigma); section 3.1: covariance estimated on a small batch). */
int fmtc_oracle_covariance(const float *x, int64_t N, int C, int64_t HW, int layout, double *mean, double *cov)
{
    if (!x || !mean || !cov || N < 1 || C < 1 || HW < 1) return ORC_EINVAL;
    double P = (double)N * (double)HW;
    for (int c = 0; c < C; c++) mean[c] = 0.0;
    for (int64_t n = 0; n < N; n++)
        for (int64_t hw = 0; hw < HW; hw++)
            for (int c = 0; c < C; c++) mean[c] += (double)x[x_index(layout, n, c, hw, C, HW)];
    for (int c = 0; c < C; c++) mean[c] /= P;
    for (size_t i = 0; i < (size_t)C * C; i++) cov[i] = 0.0;
    double *d = (double *)malloc(sizeof(double) * (size_t)C);
    if (!d) return ORC_ENOMEM;
    for (int64_t n = 0; n < N; n++)
        for (int64_t hw = 0; hw < HW; hw++) {
            for (int c = 0; c < C; c++) d[c] = (double)x[x_index(layout, n, c, hw, C, HW)] - mean[c];
            for (int i = 0; i < C; i++)
                for (int j = 0; j < C; j++) cov[(size_t)i * C + j] += d[i] * d[j];
        }
    for (size_t i = 0; i < (size_t)C * C; i++) cov[i] /= P;
    free(d);
    return ORC_OK;
}

/* PCA basis of a covariance matrix: rows of T are the eigenvectors of cov in
 * order of descending eigenvalue (section 3: the orthonormal T that
 * diagonalises Sigma; T^-1 = T^T).  Sign: the entry of largest magnitude in
 * each row is positive (first one on ties).  T is returned in fp64. */
int fmtc_oracle_pca(const double *cov, int C, double *T, double *eig)
{
    if (!cov || !T || !eig || C < 1) return ORC_EINVAL;
    double *a = (double *)malloc(sizeof(double) * (size_t)C * C);
    double *v = (double *)malloc(sizeof(double) * (size_t)C * C);
    int *order = (int *)malloc(sizeof(int) * (size_t)C);
    if (!a || !v || !order) { free(a); free(v); free(order); return ORC_ENOMEM; }
    memcpy(a, cov, sizeof(double) * (size_t)C * C);
    jacobi_eigh(a, v, C);
    for (int i = 0; i < C; i++) order[i] = i;
    /* stable insertion sort, descending eigenvalue */
    for (int i = 1; i < C; i++) {
        int o = order[i];
        double e = a[(size_t)o * C + o];
        int j = i - 1;
        while (j >= 0 && a[(size_t)order[j] * C + order[j]] < e) { order[j + 1] = order[j]; j--; }
        order[j + 1] = o;
    }
    for (int k = 0; k < C; k++) {
        int col = order[k];
        eig[k] = a[(size_t)col * C + col];
        int arg = 0;
        double best = -1.0;
        for (int c = 0; c < C; c++) {
            double m = fabs(v[(size_t)c * C + col]);
            if (m > best) { best = m; arg = c; }
        }
        double sgn = v[(size_t)arg * C + col] < 0.0 ? -1.0 : 1.0;
        for (int c = 0; c < C; c++) T[(size_t)k * C + c] = sgn * v[(size_t)c * C + col];
    }
    free(a); free(v); free(order);
    return ORC_OK;
}

/* y = T (x - mu) for every 1x1xC block, fp64 (section 3).  y is [P][C], pixel
 * major in logical (n, h, w) order, coefficient minor. */
int fmtc_oracle_project(const float *x, int64_t N, int C, int64_t HW, int layout,
                        const float *T, const float *mu, double *y)
{
    if (!x || !T || !mu || !y || N < 1 || C < 1 || HW < 1) return ORC_EINVAL;
    double *d = (double *)malloc(sizeof(double) * (size_t)C);
    if (!d) return ORC_ENOMEM;
    for (int64_t n = 0; n < N; n++)
        for (int64_t hw = 0; hw < HW; hw++) {
            size_t p = (size_t)n * (size_t)HW + (size_t)hw;
            for (int c = 0; c < C; c++) d[c] = (double)x[x_index(layout, n, c, hw, C, HW)] - (double)mu[c];
            for (int k = 0; k < C; k++) {
                double acc = 0.0;
                for (int c = 0; c < C; c++) acc += (double)T[(size_t)k * C + c] * d[c];
                y[p * (size_t)C + k] = acc;
            }
        }
    free(d);
    return ORC_OK;
}

/* Full fit (section 3.1 "Linear transform" and "Quantization"): mean,
 * covariance, PCA, rounding of T and mu to fp32, and the dynamic range
 * A = max |y_0| over the calibration pixels, y_0 being the coefficient of the
 * highest-variance component computed with the rounded T and mu. */
int fmtc_oracle_fit(const float *x, int64_t N, int C, int64_t HW, int layout,
                    float *T, float *mu, double *eig, float *range_A)
{
    if (!x || !T || !mu || !eig || !range_A || N < 1 || C < 1 || HW < 1) return ORC_EINVAL;
    double *mean = (double *)malloc(sizeof(double) * (size_t)C);
    double *cov = (double *)malloc(sizeof(double) * (size_t)C * C);
    double *Td = (double *)malloc(sizeof(double) * (size_t)C * C);
    if (!mean || !cov || !Td) { free(mean); free(cov); free(Td); return ORC_ENOMEM; }
    int rc = fmtc_oracle_covariance(x, N, C, HW, layout, mean, cov);
    if (rc == ORC_OK) rc = fmtc_oracle_pca(cov, C, Td, eig);
    if (rc == ORC_OK) {
        for (size_t i = 0; i < (size_t)C * C; i++) T[i] = (float)Td[i];
        for (int c = 0; c < C; c++) mu[c] = (float)mean[c];
        double amax = 0.0;
        for (int64_t n = 0; n < N; n++)
            for (int64_t hw = 0; hw < HW; hw++) {
                double acc = 0.0;
                for (int c = 0; c < C; c++)
                    acc += (double)T[c] * ((double)x[x_index(layout, n, c, hw, C, HW)] - (double)mu[c]);
                if (fabs(acc) > amax) amax = fabs(acc);
            }
        *range_A = (float)amax;
    }
    free(mean); free(cov); free(Td);
    return rc;
}

/* Dynamic range of the leading component over the pixels of a given tensor:
 * A = max |t0 . (x - mu)| with the fp32 row t0 and mean (section 3.1
 * "Quantization").  Serves a calibration whose statistics come from several
 * tensors while the range is measured on one of them. */
int fmtc_oracle_range(const float *x, int64_t N, int C, int64_t HW, int layout, const float *t0, const float *mu,
                      float *range_A)
{
    if (!x || !t0 || !mu || !range_A || N < 1 || C < 1 || HW < 1) return ORC_EINVAL;
    double amax = 0.0;
    for (int64_t n = 0; n < N; n++)
        for (int64_t hw = 0; hw < HW; hw++) {
            double acc = 0.0;
            for (int c = 0; c < C; c++)
                acc += (double)t0[c] * ((double)x[x_index(layout, n, c, hw, C, HW)] - (double)mu[c]);
            if (fabs(acc) > amax) amax = fabs(acc);
        }
    *range_A = (float)amax;
    return ORC_OK;
}

/* Projection with the least significant components dropped (section 4
 * "Ablation study"): only the `keep` leading coefficients are computed; a
 * dropped coefficient is 0 (its symbol is then the zero level).  y is [P][C]. */
int fmtc_oracle_project_keep(const float *x, int64_t N, int C, int64_t HW, int layout,
                             const float *T, const float *mu, int keep, double *y)
{
    if (!x || !T || !mu || !y || N < 1 || C < 1 || HW < 1 || keep < 1 || keep > C) return ORC_EINVAL;
    double *d = (double *)malloc(sizeof(double) * (size_t)C);
    if (!d) return ORC_ENOMEM;
    for (int64_t n = 0; n < N; n++)
        for (int64_t hw = 0; hw < HW; hw++) {
            size_t p = (size_t)n * (size_t)HW + (size_t)hw;
            for (int c = 0; c < C; c++) d[c] = (double)x[x_index(layout, n, c, hw, C, HW)] - (double)mu[c];
            for (int k = 0; k < keep; k++) {
                double acc = 0.0;
                for (int c = 0; c < C; c++) acc += (double)T[(size_t)k * C + c] * d[c];
                y[p * (size_t)C + k] = acc;
            }
            for (int k = keep; k < C; k++) y[p * (size_t)C + k] = 0.0;
        }
    free(d);
    return ORC_OK;
}

/* ------------------------------------------------------------ quantizer */

/* Step of the b-bit mid-tread quantizer whose positive range 2^(b-1)-1 levels
 * spans the dynamic range A of the highest-variance component (section 3.1
 * "Quantization").  A degenerate range (A == 0) takes step 1. */
float fmtc_oracle_delta(float range_A, int bits)
{
    if (!(range_A > 0.0f)) return 1.0f;
    return (float)((double)range_A / (double)((1 << (bits - 1)) - 1));
}

/* Uniform scalar quantizer Q_Delta (section 3): level q = round-half-even(y/Delta)
 * clamped to [-2^(b-1), 2^(b-1)-1]; symbol s = q + 2^(b-1).  margin (optional)
 * receives the distance of y/Delta to the nearest rounding boundary, in steps. */
int fmtc_oracle_quantize(const double *y, int64_t count, float delta, int bits, uint8_t *sym, double *margin)
{
    if (!y || !sym || count < 0 || bits < 2 || bits > 8 || !(delta > 0.0f)) return ORC_EINVAL;
    double half = (double)(1 << (bits - 1));
    for (int64_t i = 0; i < count; i++) {
        double t = y[i] / (double)delta;
        double r = nearbyint(t); /* default rounding mode: ties to even */
        if (r < -half) r = -half;
        if (r > half - 1.0) r = half - 1.0;
        sym[i] = (uint8_t)(int)(r + half);
        if (margin) margin[i] = fabs((t - floor(t)) - 0.5);
    }
    return ORC_OK;
}

/* ------------------------------------------------- statistics and Huffman */

/* Symbol counts over the whole tensor (section 3.1 "Variable length coding"). */
int fmtc_oracle_histogram(const uint8_t *sym, int64_t count, int bits, uint64_t *hist)
{
    if (!sym || !hist || count < 0 || bits < 2 || bits > 8) return ORC_EINVAL;
    int K = 1 << bits;
    for (int s = 0; s < MAX_SYMS; s++) hist[s] = 0;
    for (int64_t i = 0; i < count; i++) {
        if (sym[i] >= K) return ORC_EINVAL;
        hist[sym[i]]++;
    }
    return ORC_OK;
}

/* H = -sum p log2 p over the used symbols (section 3.1). */
double fmtc_oracle_entropy(const uint64_t *hist, int K)
{
    double total = 0.0, h = 0.0;
    for (int s = 0; s < K; s++) total += (double)hist[s];
    if (total == 0.0) return 0.0;
    for (int s = 0; s < K; s++)
        if (hist[s]) {
            double p = (double)hist[s] / total;
            h -= p * log2(p);
        }
    return h;
}

/* Code lengths of a Huffman code (optimal prefix code, unlimited length) for
 * the counts hist[0..K).  Construction: leaves sorted ascending by (count,
 * symbol); repeatedly merge the two lightest nodes, a leaf winning over an
 * internal node of equal weight and internal nodes leaving in creation order.
 * Unused symbols get length 0; a lone used symbol gets length 1. */
int fmtc_oracle_huffman_lengths(const uint64_t *hist, int K, uint8_t *len)
{
    if (!hist || !len || K < 1 || K > MAX_SYMS) return ORC_EINVAL;
    int leaf_sym[MAX_SYMS];
    uint64_t weight[2 * MAX_SYMS];
    int parent[2 * MAX_SYMS];
    int depth[2 * MAX_SYMS];
    int n = 0;
    for (int s = 0; s < K; s++) len[s] = 0;
    for (int s = 0; s < K; s++)
        if (hist[s]) {
            /* insertion keeps (count, symbol) ascending because s only grows */
            int j = n - 1;
            while (j >= 0 && hist[leaf_sym[j]] > hist[s]) { leaf_sym[j + 1] = leaf_sym[j]; j--; }
            leaf_sym[j + 1] = s;
            n++;
        }
    if (n == 0) return ORC_EINVAL;
    if (n == 1) { len[leaf_sym[0]] = 1; return ORC_OK; }
    for (int i = 0; i < n; i++) weight[i] = hist[leaf_sym[i]];
    int next_leaf = 0, next_int = n, made = n; /* internal nodes live at n .. 2n-2 */
    for (int m = 0; m < n - 1; m++) {
        int pick[2];
        for (int t = 0; t < 2; t++) {
            int have_leaf = next_leaf < n, have_int = next_int < made;
            if (have_leaf && (!have_int || weight[next_leaf] <= weight[next_int])) pick[t] = next_leaf++;
            else pick[t] = next_int++;
        }
        weight[made] = weight[pick[0]] + weight[pick[1]];
        parent[pick[0]] = made;
        parent[pick[1]] = made;
        made++;
    }
    int root = made - 1;
    depth[root] = 0;
    for (int node = root - 1; node >= 0; node--) depth[node] = depth[parent[node]] + 1;
    for (int i = 0; i < n; i++) {
        if (depth[i] > MAX_LEN) return ORC_EINVAL;
        len[leaf_sym[i]] = (uint8_t)depth[i];
    }
    return ORC_OK;
}

/* Code lengths of a table made before the tensors it will code are known
 * (section 3.1 names a Huffman code and leaves open when its table is made; a
 * coder that emits bits as the values arrive cannot take it from the tensor
 * itself).  Reading: the counts are those of a calibration tensor's symbols,
 * and one is added to every symbol of the alphabet, so that any symbol a
 * later tensor holds has a code.  Huffman lengths of those counts. */
int fmtc_oracle_static_lengths(const uint64_t *calib_hist, int K, uint8_t *len)
{
    if (!calib_hist || !len || K < 2 || K > MAX_SYMS) return ORC_EINVAL;
    uint64_t smoothed[MAX_SYMS];
    for (int s = 0; s < K; s++) smoothed[s] = calib_hist[s] + 1;
    return fmtc_oracle_huffman_lengths(smoothed, K, len);
}

/* Canonical code words for given lengths: used symbols ordered by (length,
 * symbol); the first gets code 0, each next one (previous + 1) shifted left by
 * the growth in length. */
int fmtc_oracle_canonical_codes(const uint8_t *len, int K, uint64_t *code)
{
    if (!len || !code || K < 1 || K > MAX_SYMS) return ORC_EINVAL;
    int first = 1, prev_len = 0;
    uint64_t prev = 0;
    for (int s = 0; s < K; s++) code[s] = 0;
    for (int l = 1; l <= MAX_LEN; l++)
        for (int s = 0; s < K; s++)
            if (len[s] == l) {
                if (first) { prev = 0; first = 0; }
                else prev = (prev + 1) << (l - prev_len);
                prev_len = l;
                code[s] = prev;
            }
    return ORC_OK;
}

/* ------------------------------------------------------------ container */
/*
 * Bit stream container (the paper only says the VLC output is accumulated in
 * external memory; the format is this build's).  Little-endian.
 *   [0,64)    header
 *   [64,320)  code length of each symbol, u8[256] (0 = unused)
 *   [320,..)  u32 chunk_off[n_chunks+1]: first payload word of every chunk
 *   align 16  u16 sub_bits[n_chunks][subs_per_chunk]: code bits of every run of
 *             64 consecutive symbols of a chunk (0 for runs past a short chunk)
 *   align 16  u32 payload[payload_words]
 * A chunk is px_per_chunk = max(1, chunk_syms / C) whole pixels; every chunk
 * starts on a word boundary, pad bits are 0.  Stream bit i is bit (i mod 32)
 * of word i/32; a code is written most significant code bit first.
 */
typedef struct {
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
} orc_header;

#define ORC_MAGIC 0x43544D46u /* bytes 'F','M','T','C' */

static size_t align16(size_t v) { return (v + 15) & ~(size_t)15; }

typedef struct {
    uint32_t px_per_chunk, n_chunks, subs_per_chunk;
    size_t off_chunk_off, off_sub_bits, off_payload;
} orc_geometry;

static int geometry(int64_t P, int C, int chunk_syms, orc_geometry *g)
{
    if (P < 1 || C < 1 || C > 1024 || chunk_syms < 64) return ORC_EINVAL;
    int64_t ppc = chunk_syms / C;
    if (ppc < 1) ppc = 1;
    int64_t nch = (P + ppc - 1) / ppc;
    if (nch > 0x7fffffff) return ORC_EINVAL;
    g->px_per_chunk = (uint32_t)ppc;
    g->n_chunks = (uint32_t)nch;
    g->subs_per_chunk = (uint32_t)((ppc * C + SUB_SYMS - 1) / SUB_SYMS);
    g->off_chunk_off = HEADER_BYTES + LEN_TABLE_BYTES;
    g->off_sub_bits = align16(g->off_chunk_off + 4 * ((size_t)nch + 1));
    g->off_payload = align16(g->off_sub_bits + 2 * (size_t)nch * g->subs_per_chunk);
    return ORC_OK;
}

/* worst-case stream size: an optimal prefix code never needs more bits in
 * total than the fixed b-bit code; each chunk adds at most one pad word. */
size_t fmtc_oracle_stream_bound(int64_t P, int C, int bits, int chunk_syms)
{
    orc_geometry g;
    if (geometry(P, C, chunk_syms, &g) != ORC_OK) return 0;
    uint64_t V = (uint64_t)P * (uint64_t)C;
    return g.off_payload + 4 * (size_t)((V * (uint64_t)bits + 31) / 32 + g.n_chunks);
}

/* Serialise symbols (pixel major, coefficient minor) with the given code. */
int fmtc_oracle_pack(const uint8_t *sym, int64_t P, int C, int bits, int chunk_syms, float delta,
                     const uint8_t *len, const uint64_t *code, uint8_t *out, size_t cap, size_t *out_bytes)
{
    orc_geometry g;
    if (!sym || !len || !code || !out || !out_bytes || bits < 2 || bits > 8) return ORC_EINVAL;
    if (geometry(P, C, chunk_syms, &g) != ORC_OK) return ORC_EINVAL;
    if (cap < g.off_payload) return ORC_EBUFSIZE;
    int K = 1 << bits;
    memset(out, 0, g.off_payload);
    uint32_t *chunk_off = (uint32_t *)(out + g.off_chunk_off);
    uint16_t *sub_bits = (uint16_t *)(out + g.off_sub_bits);
    uint32_t *payload = (uint32_t *)(out + g.off_payload);
    size_t cap_words = (cap - g.off_payload) / 4;
    uint64_t word = 0, total_bits = 0;
    for (uint32_t ch = 0; ch < g.n_chunks; ch++) {
        int64_t p0 = (int64_t)ch * g.px_per_chunk;
        int64_t p1 = p0 + g.px_per_chunk;
        if (p1 > P) p1 = P;
        int64_t s0 = p0 * C, s1 = p1 * C;
        uint64_t bitpos = 0; /* within the chunk */
        chunk_off[ch] = (uint32_t)word;
        for (int64_t i = s0; i < s1; i++) {
            int s = sym[i];
            if (s >= K || len[s] == 0) return ORC_EINVAL;
            int l = len[s];
            for (int b = l - 1; b >= 0; b--) { /* most significant code bit first */
                size_t w = (size_t)word + (size_t)(bitpos >> 5);
                if (w >= cap_words) return ORC_EBUFSIZE;
                if ((bitpos & 31) == 0) payload[w] = 0;
                if ((code[s] >> b) & 1) payload[w] |= (uint32_t)1 << (bitpos & 31);
                bitpos++;
            }
            sub_bits[(size_t)ch * g.subs_per_chunk + (size_t)((i - s0) / SUB_SYMS)] += (uint16_t)l;
        }
        total_bits += bitpos;
        word += (bitpos + 31) >> 5;
        if (word > 0xffffffffu) return ORC_EINVAL;
    }
    chunk_off[g.n_chunks] = (uint32_t)word;
    orc_header h;
    memset(&h, 0, sizeof h);
    h.magic = ORC_MAGIC; h.version = 1; h.bits = (uint8_t)bits; h.C = (uint32_t)C;
    h.px_per_chunk = g.px_per_chunk; h.P = (uint64_t)P; h.n_chunks = g.n_chunks; h.sub_syms = SUB_SYMS;
    h.delta = delta; h.subs_per_chunk = g.subs_per_chunk; h.payload_words = word; h.payload_bits = total_bits;
    memcpy(out, &h, sizeof h);
    memcpy(out + HEADER_BYTES, len, (size_t)K);
    *out_bytes = g.off_payload + 4 * (size_t)word;
    return ORC_OK;
}

/* Variable length decoder: validates the container, then reads every chunk
 * bit by bit with the canonical code rebuilt from the length table. */
int fmtc_oracle_unpack(const uint8_t *in, size_t bytes, int64_t P, int C, int bits,
                       uint8_t *sym, float *delta_out, uint64_t *payload_bits_out)
{
    if (!in || !sym || bits < 2 || bits > 8) return ORC_EINVAL;
    if (bytes < HEADER_BYTES + LEN_TABLE_BYTES) return ORC_ECORRUPT;
    orc_header h;
    memcpy(&h, in, sizeof h);
    if (h.magic != ORC_MAGIC || h.version != 1 || h.bits != bits || h.C != (uint32_t)C ||
        h.P != (uint64_t)P || h.sub_syms != SUB_SYMS || h.px_per_chunk < 1 || !(h.delta > 0.0f))
        return ORC_ECORRUPT;
    orc_geometry g;
    /* px_per_chunk fixes the geometry: rebuild it from a chunk_syms that reproduces it */
    if (geometry(P, C, (int)((int64_t)h.px_per_chunk * C < 64 ? 64 : (int64_t)h.px_per_chunk * C), &g) != ORC_OK)
        return ORC_ECORRUPT;
    if (g.px_per_chunk != h.px_per_chunk || g.n_chunks != h.n_chunks || g.subs_per_chunk != h.subs_per_chunk)
        return ORC_ECORRUPT;
    if (bytes < g.off_payload || (bytes - g.off_payload) / 4 < h.payload_words) return ORC_ECORRUPT;
    const uint8_t *len = in + HEADER_BYTES;
    const uint32_t *chunk_off = (const uint32_t *)(in + g.off_chunk_off);
    const uint16_t *sub_bits = (const uint16_t *)(in + g.off_sub_bits);
    const uint32_t *payload = (const uint32_t *)(in + g.off_payload);
    int K = 1 << bits;
    /* code table checks: lengths in range, Kraft equality (or the lone symbol case) */
    int used = 0;
    uint64_t kraft = 0; /* in units of 2^-MAX_LEN */
    uint32_t count[MAX_LEN + 1];
    memset(count, 0, sizeof count);
    for (int s = 0; s < MAX_SYMS; s++) {
        if (len[s] > MAX_LEN || (s >= K && len[s] != 0)) return ORC_ECORRUPT;
        if (len[s]) { used++; count[len[s]]++; kraft += (uint64_t)1 << (MAX_LEN - len[s]); }
    }
    if (used == 0) return ORC_ECORRUPT;
    if (used == 1) { if (count[1] != 1) return ORC_ECORRUPT; }
    else if (kraft != ((uint64_t)1 << MAX_LEN)) return ORC_ECORRUPT;
    uint64_t code[MAX_SYMS];
    fmtc_oracle_canonical_codes(len, K, code);
    uint64_t first_code[MAX_LEN + 1];
    int first_rank[MAX_LEN + 1];
    int by_rank[MAX_SYMS];
    int r = 0;
    for (int l = 1; l <= MAX_LEN; l++) {
        first_rank[l] = r;
        first_code[l] = 0;
        int seen = 0;
        for (int s = 0; s < K; s++)
            if (len[s] == l) {
                if (!seen) { first_code[l] = code[s]; seen = 1; }
                by_rank[r++] = s;
            }
    }
    if (chunk_off[0] != 0 || chunk_off[g.n_chunks] != h.payload_words) return ORC_ECORRUPT;
    uint64_t total_bits = 0;
    for (uint32_t ch = 0; ch < g.n_chunks; ch++) {
        int64_t p0 = (int64_t)ch * g.px_per_chunk;
        int64_t p1 = p0 + g.px_per_chunk;
        if (p1 > P) p1 = P;
        int64_t s0 = p0 * C, s1 = p1 * C;
        if (chunk_off[ch + 1] < chunk_off[ch] || chunk_off[ch + 1] > h.payload_words) return ORC_ECORRUPT;
        uint64_t avail = ((uint64_t)chunk_off[ch + 1] - chunk_off[ch]) * 32;
        const uint32_t *w = payload + chunk_off[ch];
        uint64_t bitpos = 0, sub_start = 0;
        for (int64_t i = s0; i < s1; i++) {
            uint64_t c = 0;
            int l = 0, found = -1;
            while (l < MAX_LEN) {
                if (bitpos >= avail) return ORC_ECORRUPT;
                c = (c << 1) | ((w[bitpos >> 5] >> (bitpos & 31)) & 1);
                bitpos++; l++;
                if (count[l] && c >= first_code[l] && c - first_code[l] < count[l]) {
                    found = by_rank[first_rank[l] + (int)(c - first_code[l])];
                    break;
                }
            }
            if (found < 0) return ORC_ECORRUPT;
            sym[i] = (uint8_t)found;
            int64_t j = i - s0;
            if ((j + 1) % SUB_SYMS == 0 || i + 1 == s1) {
                if (sub_bits[(size_t)ch * g.subs_per_chunk + (size_t)(j / SUB_SYMS)] != bitpos - sub_start)
                    return ORC_ECORRUPT;
                sub_start = bitpos;
            }
        }
        if ((bitpos + 31) / 32 * 32 != avail) return ORC_ECORRUPT;
        for (uint64_t b = bitpos; b < avail; b++)
            if ((w[b >> 5] >> (b & 31)) & 1) return ORC_ECORRUPT;
        total_bits += bitpos;
    }
    if (total_bits != h.payload_bits) return ORC_ECORRUPT;
    if (delta_out) *delta_out = h.delta;
    if (payload_bits_out) *payload_bits_out = total_bits;
    return ORC_OK;
}

/* ------------------------------------------------ inverse quantizer / transform */

/* y_hat = Delta (s - 2^(b-1)); x_hat = T^T y_hat + mu (section 3: inverse
 * quantizer, then inverse transform; T^-1 = T^T).  No non-linearity, no clipping. */
int fmtc_oracle_reconstruct(const uint8_t *sym, int64_t N, int C, int64_t HW, int layout, int bits, float delta,
                            const float *T, const float *mu, double *xhat)
{
    if (!sym || !T || !mu || !xhat || N < 1 || C < 1 || HW < 1 || bits < 2 || bits > 8) return ORC_EINVAL;
    double half = (double)(1 << (bits - 1));
    double *yh = (double *)malloc(sizeof(double) * (size_t)C);
    if (!yh) return ORC_ENOMEM;
    for (int64_t n = 0; n < N; n++)
        for (int64_t hw = 0; hw < HW; hw++) {
            size_t p = (size_t)n * (size_t)HW + (size_t)hw;
            for (int k = 0; k < C; k++) yh[k] = (double)delta * ((double)sym[p * (size_t)C + k] - half);
            for (int c = 0; c < C; c++) {
                double acc = 0.0;
                for (int k = 0; k < C; k++) acc += (double)T[(size_t)k * C + c] * yh[k];
                xhat[x_index(layout, n, c, hw, C, HW)] = acc + (double)mu[c];
            }
        }
    free(yh);
    return ORC_OK;
}

/* Reconstruction from the `keep` leading components only (section 4 "Ablation
 * study"): x_hat = sum_{k < keep} T[k] y_hat[k] + mu; the symbols of the dropped
 * coefficients are not looked at. */
int fmtc_oracle_reconstruct_keep(const uint8_t *sym, int64_t N, int C, int64_t HW, int layout, int bits, float delta,
                                 const float *T, const float *mu, int keep, double *xhat)
{
    if (!sym || !T || !mu || !xhat || N < 1 || C < 1 || HW < 1 || bits < 2 || bits > 8 || keep < 1 || keep > C)
        return ORC_EINVAL;
    double half = (double)(1 << (bits - 1));
    for (int64_t n = 0; n < N; n++)
        for (int64_t hw = 0; hw < HW; hw++) {
            size_t p = (size_t)n * (size_t)HW + (size_t)hw;
            for (int c = 0; c < C; c++) {
                double acc = 0.0;
                for (int k = 0; k < keep; k++)
                    acc += (double)T[(size_t)k * C + c] * ((double)delta * ((double)sym[p * (size_t)C + k] - half));
                xhat[x_index(layout, n, c, hw, C, HW)] = acc + (double)mu[c];
            }
        }
    return ORC_OK;
}

/* ------------------------------------------- 8-bit basis and 8-bit activations */

/* Section 3.1 "Linear transform" stores the PCA matrix at 8 bits, and the
 * hardware of section 5 moves 8-bit activations.  The arithmetic below is the
 * integer reading of y = T (x - mu), Q, Q^-1 and x_hat = T^T y_hat + mu for
 *   x   = s_x * xq,        xq unsigned 8-bit (post-activation maps),
 *   T   = s_T * Tq,        Tq = clamp(rne(T / s_T), -127, 127), s_T = (float)(max|T| / 127),
 *   mu  = s_x * mf / 256,  mf = rne(256 mu / s_x)   (the mean with 8 fraction bits on the activations' grid).
 * Sums are exact integers; every rounding decision is one correctly rounded
 * fp64 operation on exact operands, so an implementation either reproduces
 * these results bit for bit or is wrong. */

/* Tq (C*C, row major), s_T and mf (C) from the fp32 basis, mean and activation scale. */
int fmtc_oracle_basis8(const float *T, const float *mu, int C, float act_scale, int8_t *Tq, float *scale_T,
                       int32_t *mean_fix)
{
    if (!T || !mu || !Tq || !scale_T || !mean_fix || C < 1 || !(act_scale > 0.0f)) return ORC_EINVAL;
    double amax = 0.0;
    for (size_t i = 0; i < (size_t)C * C; i++)
        if (fabs((double)T[i]) > amax) amax = fabs((double)T[i]);
    float sT = (float)(amax / 127.0);
    if (!(sT > 0.0f)) sT = 1.0f;
    for (size_t i = 0; i < (size_t)C * C; i++) {
        double r = nearbyint((double)T[i] / (double)sT);
        if (r > 127.0) r = 127.0;
        if (r < -127.0) r = -127.0;
        Tq[i] = (int8_t)(int)r;
    }
    for (int c = 0; c < C; c++) mean_fix[c] = (int32_t)nearbyint((double)mu[c] / (double)act_scale * 256.0);
    *scale_T = sT;
    return ORC_OK;
}

/* Symbols of 8-bit activations under the 8-bit basis: for every pixel and
 * coefficient k, n = 256 sum_c Tq[k][c] xq[c] - sum_c Tq[k][c] mf[c] (an exact
 * integer, = 256 y / (s_T s_x)), level = rne(n * g) with the single fp64 factor
 * g = (s_T s_x) / (256 Delta), clamped; symbol = level + 2^(b-1).  [P][C]. */
int fmtc_oracle_quantize_u8(const uint8_t *xq, int64_t N, int C, int64_t HW, int layout, const int8_t *Tq,
                            float scale_T, const int32_t *mean_fix, float act_scale, float delta, int bits,
                            uint8_t *sym)
{
    if (!xq || !Tq || !mean_fix || !sym || N < 1 || C < 1 || HW < 1 || bits < 2 || bits > 8) return ORC_EINVAL;
    if (!(scale_T > 0.0f) || !(act_scale > 0.0f) || !(delta > 0.0f)) return ORC_EINVAL;
    const double g = ((double)scale_T * (double)act_scale) / (256.0 * (double)delta);
    const double half = (double)(1 << (bits - 1));
    for (int64_t n = 0; n < N; n++)
        for (int64_t hw = 0; hw < HW; hw++) {
            size_t p = (size_t)n * (size_t)HW + (size_t)hw;
            for (int k = 0; k < C; k++) {
                int64_t dot = 0, off = 0;
                for (int c = 0; c < C; c++) {
                    dot += (int64_t)Tq[(size_t)k * C + c] * (int64_t)xq[x_index(layout, n, c, hw, C, HW)];
                    off += (int64_t)Tq[(size_t)k * C + c] * (int64_t)mean_fix[c];
                }
                double r = nearbyint((double)(256 * dot - off) * g);
                if (r < -half) r = -half;
                if (r > half - 1.0) r = half - 1.0;
                sym[p * (size_t)C + k] = (uint8_t)(int)(r + half);
            }
        }
    return ORC_OK;
}

/* 8-bit activations back from symbols: with levels q = s - 2^(b-1) and the exact
 * integer m = sum_k Tq[k][c] q[k], the value on the activations' grid with 8
 * fraction bits is v = fma(m, h, mf[c]), h = (s_T Delta 256) / s_x (one fused
 * fp64 operation), and xq_hat = clamp(rne(v / 256), 0, 255). */
int fmtc_oracle_reconstruct_u8(const uint8_t *sym, int64_t N, int C, int64_t HW, int layout, const int8_t *Tq,
                               float scale_T, const int32_t *mean_fix, float act_scale, float delta, int bits,
                               uint8_t *xq_hat)
{
    if (!sym || !Tq || !mean_fix || !xq_hat || N < 1 || C < 1 || HW < 1 || bits < 2 || bits > 8) return ORC_EINVAL;
    if (!(scale_T > 0.0f) || !(act_scale > 0.0f) || !(delta > 0.0f)) return ORC_EINVAL;
    const double h = ((double)scale_T * (double)delta * 256.0) / (double)act_scale;
    const int halfk = 1 << (bits - 1);
    for (int64_t n = 0; n < N; n++)
        for (int64_t hw = 0; hw < HW; hw++) {
            size_t p = (size_t)n * (size_t)HW + (size_t)hw;
            for (int c = 0; c < C; c++) {
                int64_t m = 0;
                for (int k = 0; k < C; k++)
                    m += (int64_t)Tq[(size_t)k * C + c] * (int64_t)((int)sym[p * (size_t)C + k] - halfk);
                double r = nearbyint(fma((double)m, h, (double)mean_fix[c]) / 256.0);
                if (r < 0.0) r = 0.0;
                if (r > 255.0) r = 255.0;
                xq_hat[x_index(layout, n, c, hw, C, HW)] = (uint8_t)(int)r;
            }
        }
    return ORC_OK;
}

/* D = (1/n) ||x - x_hat||^2 (section 3). */
double fmtc_oracle_mse(const float *x, const double *xhat, int64_t count)
{
    double acc = 0.0;
    for (int64_t i = 0; i < count; i++) {
        double d = (double)x[i] - xhat[i];
        acc += d * d;
    }
    return count ? acc / (double)count : 0.0;
}

/* ------------------------------------------------ whole encode / decode */

/* project -> quantize -> histogram -> Huffman -> pack.  Optional outputs:
 * sym [P*C], margin [P*C], hist [256]. */
int fmtc_oracle_encode(const float *x, int64_t N, int C, int64_t HW, int layout, const float *T, const float *mu,
                       float delta, int bits, int chunk_syms, uint8_t *out, size_t cap, size_t *out_bytes,
                       uint8_t *sym_out, double *margin_out, uint64_t *hist_out)
{
    int64_t P = N * HW;
    size_t V = (size_t)P * (size_t)C;
    double *y = (double *)malloc(sizeof(double) * V);
    uint8_t *sym = sym_out ? sym_out : (uint8_t *)malloc(V);
    uint64_t hist[MAX_SYMS], code[MAX_SYMS];
    uint8_t len[MAX_SYMS];
    int rc = (y && sym) ? ORC_OK : ORC_ENOMEM;
    if (rc == ORC_OK) rc = fmtc_oracle_project(x, N, C, HW, layout, T, mu, y);
    if (rc == ORC_OK) rc = fmtc_oracle_quantize(y, (int64_t)V, delta, bits, sym, margin_out);
    if (rc == ORC_OK) rc = fmtc_oracle_histogram(sym, (int64_t)V, bits, hist);
    if (rc == ORC_OK) rc = fmtc_oracle_huffman_lengths(hist, 1 << bits, len);
    if (rc == ORC_OK) rc = fmtc_oracle_canonical_codes(len, 1 << bits, code);
    if (rc == ORC_OK) rc = fmtc_oracle_pack(sym, P, C, bits, chunk_syms, delta, len, code, out, cap, out_bytes);
    if (rc == ORC_OK && hist_out) memcpy(hist_out, hist, sizeof hist);
    free(y);
    if (!sym_out) free(sym);
    return rc;
}

/* unpack -> dequantize -> inverse transform. */
int fmtc_oracle_decode(const uint8_t *in, size_t bytes, int64_t N, int C, int64_t HW, int layout, int bits,
                       const float *T, const float *mu, double *xhat, uint8_t *sym_out)
{
    int64_t P = N * HW;
    size_t V = (size_t)P * (size_t)C;
    uint8_t *sym = sym_out ? sym_out : (uint8_t *)malloc(V);
    if (!sym) return ORC_ENOMEM;
    float delta = 0.0f;
    int rc = fmtc_oracle_unpack(in, bytes, P, C, bits, sym, &delta, NULL);
    if (rc == ORC_OK) rc = fmtc_oracle_reconstruct(sym, N, C, HW, layout, bits, delta, T, mu, xhat);
    if (!sym_out) free(sym);
    return rc;
}
