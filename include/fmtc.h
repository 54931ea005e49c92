/*
 * fmtc.h -- C ABI of the feature-map transform codec for AMD MI355X (gfx950).
 *
 * The codec is the encoder/decoder chain of "Feature Map Transform Coding for
 * Energy-Efficient CNN Inference" (arXiv 1905.10830):
 *
 *   encode (section 3; section 3.1 "Implementation"): every 1x1xC block x of an
 *   activation tensor is transformed, y = T (x - mu), with the orthonormal PCA
 *   basis T of the channel covariance; y is quantized by a uniform scalar
 *   quantizer with one step Delta for all coefficients; the levels are coded
 *   with a Huffman code built from the tensor's own symbol histogram and the
 *   bits are written to memory.
 *   decode: variable length decoding, levels scaled back by Delta, inverse
 *   transform x_hat = T^T y_hat + mu.  No non-linearity is applied.
 *
 * Conventions
 *   - Plain C types only.  d_* pointers are DEVICE pointers owned by the caller,
 *     h_* pointers are HOST pointers owned by the caller.  hip_stream is a
 *     hipStream_t passed as void* (NULL = the default stream).
 *   - Logical tensor dims are always (N, C, H, W); `layout` selects the storage:
 *     FMTC_NHWC = [N][H][W][C] contiguous, FMTC_NCHW = [N][C][H][W] contiguous.
 *     P = N*H*W pixels, V = P*C values.
 *   - Symbols: level q in [-2^(b-1), 2^(b-1)-1] is stored as s = q + 2^(b-1),
 *     one byte each, pixel major in logical (n,h,w) order, coefficient minor.
 *   - Every call returns a status and never throws.  Argument errors are found
 *     on the host before any launch; fmtc_last_error() gives the text for the
 *     calling thread.  All hot-path calls are asynchronous on hip_stream and
 *     allocate nothing: scratch comes from the caller's workspace.
 *   - Limits: 1 <= C <= 1024, 2 <= bits <= 8, 64 <= chunk_syms <= 4096, V < 2^32.
 *   - Two calls may overlap only if they use different workspaces and outputs.
 *
 * Stream container (little endian; this library's own format, the paper leaves
 * it open):
 *   [0,64)    header: u32 magic "FMTC", u16 version=1, u8 bits, u8 0, u32 C,
 *             u32 px_per_chunk, u64 P, u32 n_chunks, u32 sub_syms=64, f32 Delta,
 *             u32 subs_per_chunk, u64 payload_words, u64 payload_bits, u64 0
 *   [64,320)  u8 code length per symbol (0 = unused symbol)
 *   [320,..)  u32 chunk_off[n_chunks+1]  first payload word of each chunk
 *   align 16  u16 sub_bits[n_chunks][subs_per_chunk]  code bits of each run of 64
 *             consecutive symbols of a chunk (lets 64 lanes decode one chunk)
 *   align 16  u32 payload[payload_words]
 *   A chunk holds px_per_chunk = max(1, chunk_syms / C) whole pixels and starts
 *   on a 32-bit word boundary; pad bits are 0.  Stream bit i is bit (i mod 32)
 *   of payload word i/32.  Codes are canonical Huffman codes (symbols ordered by
 *   (length, symbol)), written most significant code bit first.
 */
#ifndef FMTC_H
#define FMTC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum fmtc_status {
    FMTC_OK = 0,
    FMTC_EINVAL = 1,   /* bad argument (null, out of range, misaligned) */
    FMTC_EBUFSIZE = 2, /* output or workspace capacity too small */
    FMTC_ECORRUPT = 3, /* stream fails validation */
    FMTC_ENOMEM = 4,   /* host or device allocation failed (basis calls only) */
    FMTC_EHIP = 5      /* a HIP runtime call failed */
} fmtc_status;

typedef enum fmtc_layout { FMTC_NCHW = 0, FMTC_NHWC = 1 } fmtc_layout;

/* Device error bits OR-ed into *d_err_flag by the decoders. */
#define FMTC_ERR_HEADER 1u  /* header does not match the arguments or the buffer size */
#define FMTC_ERR_TABLE 2u   /* code length table is not a complete prefix code */
#define FMTC_ERR_OFFSETS 4u /* chunk offsets not monotone or past the payload */
#define FMTC_ERR_CODE 8u    /* bits that match no code word, or a read past the payload */

/* Basis handle: T (CxC, row k = k-th principal component), mu (C), the
 * eigenvalues and the dynamic range A.  Owned by the library; holds small
 * device copies of T in the operand order of the kernels. */
typedef struct fmtc_basis fmtc_basis;

/* ---- offline: the transform (section 3.1 "Linear transform", "Quantization") ----
 * Fits the PCA basis on a calibration tensor resident on the device: channel
 * mean and covariance (fp64 accumulation on the GPU), symmetric eigen-
 * decomposition in fp64 on the host, rows ordered by descending eigenvalue and
 * signed so that the largest-magnitude entry of each row is positive, T and mu
 * rounded to fp32; A = max |y_0| over the calibration pixels (y_0: coefficient
 * of the highest-variance component).  Synchronises the stream.  *out must be
 * released with fmtc_basis_destroy. */
fmtc_status fmtc_fit_basis(const float *d_x, int64_t N, int C, int H, int W, fmtc_layout layout, void *hip_stream,
                           fmtc_basis **out);

/* Calibration over several tensors (section 3.1 "Linear transform": the
 * covariance comes from a small batch and may be updated online).  A fit state
 * holds, on the host in fp64, the pixel count, the channel mean and the centred
 * second moments of everything it has seen.  fmtc_fit_state_update adds one
 * device tensor (moments accumulated on the GPU as in fmtc_fit_basis, merged by
 * the exact rule for the union of two sample sets; synchronises the stream).
 * fmtc_fit_state_basis makes a basis exactly as fmtc_fit_basis would from the
 * concatenation of all tensors seen (up to rounding order), except that the
 * dynamic range A is measured over the pixels of the tensor passed here
 * (d_x, typically the latest batch): a maximum under a basis that changes with
 * every update cannot be carried along.  The state is not consumed; more updates
 * and further bases may follow.  Errors: FMTC_EINVAL for NULL or mismatching
 * arguments and for a state that has seen nothing. */
typedef struct fmtc_fit_state fmtc_fit_state;
fmtc_status fmtc_fit_state_create(int C, fmtc_fit_state **out);
fmtc_status fmtc_fit_state_update(fmtc_fit_state *state, const float *d_x, int64_t N, int C, int H, int W,
                                  fmtc_layout layout, void *hip_stream);
fmtc_status fmtc_fit_state_basis(const fmtc_fit_state *state, const float *d_x, int64_t N, int C, int H, int W,
                                 fmtc_layout layout, void *hip_stream, fmtc_basis **out);
int64_t fmtc_fit_state_count(const fmtc_fit_state *state);
void fmtc_fit_state_destroy(fmtc_fit_state *state);

/* Truncated basis (section 4 "Ablation study": the least significant
 * principal components are dropped).  *out is a new handle whose rows keep..C-1
 * of T are zero, everything else (mean, A, eigenvalues) as in `basis`; 1 <= keep
 * <= C.  With it every entry point works unchanged: a dropped coefficient is 0,
 * its symbol the zero level 2^(bits-1), and the reconstruction is the sum over
 * the kept components plus the mean.  The container keeps C symbols per pixel,
 * so a dropped coefficient still costs its (short) code word.  The kernels
 * skip the dropped rows in the units they work in (projection: tiles of 32 or
 * groups of 128 coefficients; decoders: steps of 16).  `basis` stays valid;
 * release both. */
fmtc_status fmtc_basis_truncate(const fmtc_basis *basis, int keep, fmtc_basis **out);

/* Builds a handle from host arrays (h_T: C*C row major, h_mu: C).  The way to
 * reuse a stored basis, and to give two implementations the same one. */
fmtc_status fmtc_basis_import(int C, const float *h_T, const float *h_mu, float range_A, fmtc_basis **out);

/* Copies the basis to host arrays; any output pointer may be NULL.
 * h_eigvals receives zeros for an imported basis. */
fmtc_status fmtc_basis_export(const fmtc_basis *basis, float *h_T, float *h_mu, double *h_eigvals, float *range_A);

int fmtc_basis_channels(const fmtc_basis *basis);
void fmtc_basis_destroy(fmtc_basis *basis);

/* Step of the b-bit quantizer: Delta = A / (2^(b-1) - 1) evaluated in fp64 and
 * rounded to fp32 (1.0 if A <= 0); the range is set by the highest-variance
 * component and shared by all coefficients (section 3.1 "Quantization"). */
float fmtc_delta(float range_A, int bits);

/* ---- sizing ---- */
/* Upper bound of the stream size in bytes (0 on invalid arguments): an optimal
 * prefix code never spends more than bits*V payload bits in total, plus one
 * pad word per chunk and the side information. */
size_t fmtc_encode_bound(int64_t P, int C, int bits, int chunk_syms);
/* Bytes of device workspace fmtc_encode / fmtc_code_symbols need (symbols,
 * histograms, code table, running chunk offsets).  256-byte aligned pointer
 * required; its contents need no initialisation and mean nothing between calls. */
size_t fmtc_workspace_size(int64_t P, int C, int bits, int chunk_syms);
/* ---- hot path ---- */
/* Calls on different HIP streams may overlap with each other and with any other
 * work on the device (each with its own workspace and outputs). */
/* Whole encoder (section 3: transform, quantizer, VLC).  Reads d_x once, writes
 * the container to d_stream_out (16-byte aligned, capacity cap >=
 * fmtc_encode_bound) and, if d_out_bytes != NULL, the stream size in bytes.
 * The Huffman table is built on the device from this tensor's histogram; the
 * call never synchronises.  Delta = fmtc_delta(A of the basis, bits). */
fmtc_status fmtc_encode(const fmtc_basis *basis, const float *d_x, int64_t N, int C, int H, int W,
                        fmtc_layout layout, int bits, int chunk_syms, void *d_stream_out, size_t cap,
                        uint64_t *d_out_bytes, void *d_workspace, size_t ws_bytes, void *hip_stream);

/* fmtc_encode for callers that cannot allocate or hand over a workspace (code
 * under HIP graph capture, serving loops, harnesses that forbid hipMalloc): the
 * same kernels and the same container, with the workspace in a device array
 * that is part of the library (FMTC_NOALLOC_SCRATCH_BYTES per GPU, held until
 * the process ends).  Accepts tensors with fmtc_workspace_size(P, C, bits,
 * chunk_syms) <= FMTC_NOALLOC_SCRATCH_BYTES (about 4.9 M values) and returns
 * FMTC_EBUFSIZE beyond that.  Calls no allocating routine; the first call on a
 * device looks the array's address up once (do that call outside a capture).
 * All calls on one GPU share that GPU's array: calls that overlap on one GPU
 * (different streams or threads) race -- keep them on one stream.  The array
 * keeps the previous call's contents; the encoder's first kernel clears what it
 * counts in, as in fmtc_encode. */
#define FMTC_NOALLOC_SCRATCH_BYTES ((size_t)6 << 20)
fmtc_status fmtc_encode_noalloc(const fmtc_basis *basis, const float *d_x, int64_t N, int C, int H, int W,
                                fmtc_layout layout, int bits, int chunk_syms, void *d_stream_out, size_t cap,
                                uint64_t *d_out_bytes, void *hip_stream);

/* Whole decoder (section 3: VLD, inverse quantizer, inverse transform).
 * `bytes` is the readable size of d_stream_in (the exact stream size or any
 * larger capacity); nothing beyond it is read.  d_xhat receives N*C*H*W floats
 * in `layout`.  *d_err_flag (device u32, required; the caller sets it to 0
 * before the call) is OR-ed with FMTC_ERR_* bits if the stream fails validation;
 * in that case d_xhat is unspecified but no access leaves the given buffers.
 * The decoder needs no workspace: every workgroup builds the decode tables from
 * the stream's code length table in LDS.  Channels-last tensors of up to 144
 * channels and some tens of MB or more are written with streaming stores
 * (they pass the device's memory-side cache instead of displacing its
 * contents; a consumer that reads the tensor at once reads it from memory). */
fmtc_status fmtc_decode(const fmtc_basis *basis, const void *d_stream_in, size_t bytes, float *d_xhat, int64_t N,
                        int C, int H, int W, fmtc_layout layout, int bits, uint32_t *d_err_flag, void *hip_stream);

/* ---- encoder with a code table fixed at calibration time ----
 * Section 3.1 ("Variable length coding") codes the quantizer output with a
 * Huffman code and says nothing on when its table is made.  fmtc_encode makes
 * it from the tensor being coded; a streaming datapath that codes values as
 * they are produced has to know the table beforehand.  fmtc_fit_table makes it
 * once from calibration data: the histogram of the calibration tensor's
 * symbols (same basis, same bit depth) with one count added to every one of
 * the 2^bits symbols, so that every symbol a later tensor can contain has a
 * code; Huffman lengths of those counts, canonical codes as in fmtc_encode.
 * The container written by fmtc_encode_static has the same format (it carries
 * the table), so fmtc_decode reads it unchanged.  For 32, 64 or 128 channels
 * with 4096-symbol chunks, and a tensor of at most four chunks per compute
 * unit of the device, projection, quantizer and bit packing run as ONE kernel
 * and the symbols never reach memory; otherwise the projection kernel is
 * followed by the packing kernel, which then skips histogram and table.
 *
 * fmtc_fit_table synchronises the stream and allocates/frees device memory
 * (calibration time, not the hot path).  fmtc_table_import takes the lengths
 * of a complete prefix code over the 2^bits symbols (h_lengths: 2^bits bytes
 * on the host, each 1..48, Kraft sum exactly 1; FMTC_EINVAL otherwise).
 * fmtc_table_export writes 256 bytes (zero beyond 2^bits).
 * fmtc_encode_static_bound: capacity that can not be exceeded whatever the
 * tensor holds (longest code for every symbol).  A smaller capacity is
 * accepted as long as it covers the side information; if the payload outgrows
 * it nothing is written past the buffer and the header is left invalid
 * (fmtc_decode then reports FMTC_ERR_HEADER). */
typedef struct fmtc_table fmtc_table;
fmtc_status fmtc_fit_table(const fmtc_basis *basis, const float *d_x, int64_t N, int C, int H, int W,
                           fmtc_layout layout, int bits, void *hip_stream, fmtc_table **out);
fmtc_status fmtc_table_import(const uint8_t *h_lengths, int bits, fmtc_table **out);
fmtc_status fmtc_table_export(const fmtc_table *table, uint8_t *h_lengths, int *bits);
void fmtc_table_destroy(fmtc_table *table);
size_t fmtc_encode_static_bound(const fmtc_table *table, int64_t P, int C, int chunk_syms);
/* Workspace: fmtc_workspace_size(P, C, bits of the table, chunk_syms). */
fmtc_status fmtc_encode_static(const fmtc_basis *basis, const fmtc_table *table, const float *d_x, int64_t N, int C,
                               int H, int W, fmtc_layout layout, int chunk_syms, void *d_stream_out, size_t cap,
                               uint64_t *d_out_bytes, void *d_workspace, size_t ws_bytes, void *hip_stream);

/* Decoder for streams written with `table` (fmtc_encode_static, or any stream
 * that carries exactly its code lengths): as fmtc_decode, but the decode
 * tables come ready-made from the handle instead of being built by every
 * workgroup from the stream.  A stream with other code lengths sets
 * FMTC_ERR_TABLE; every other check of fmtc_decode still applies. */
fmtc_status fmtc_decode_static(const fmtc_basis *basis, const fmtc_table *table, const void *d_stream_in, size_t bytes,
                               float *d_xhat, int64_t N, int C, int H, int W, fmtc_layout layout,
                               uint32_t *d_err_flag, void *hip_stream);

/* ---- staged entry points (the same kernels, cut at the symbol boundary) ---- */
/* Transform + quantizer + histogram only (section 3: y = T(x-mu), Q_Delta).
 * d_syms: P*C bytes; d_hist: 256 u32 counts (may be NULL). */
fmtc_status fmtc_quantize(const fmtc_basis *basis, const float *d_x, int64_t N, int C, int H, int W,
                          fmtc_layout layout, int bits, uint8_t *d_syms, uint32_t *d_hist, void *d_workspace,
                          size_t ws_bytes, void *hip_stream);

/* Histogram + Huffman table + bit packing of given symbols (section 3.1
 * "Variable length coding").  d_syms: P*C bytes, every value < 2^bits. */
fmtc_status fmtc_code_symbols(const uint8_t *d_syms, int64_t P, int C, int bits, int chunk_syms, float delta,
                              void *d_stream_out, size_t cap, uint64_t *d_out_bytes, void *d_workspace,
                              size_t ws_bytes, void *hip_stream);

/* Variable length decoder only: stream -> P*C symbol bytes. */
fmtc_status fmtc_decode_symbols(const void *d_stream_in, size_t bytes, int64_t P, int C, int bits, uint8_t *d_syms,
                                uint32_t *d_err_flag, void *hip_stream);

/* Parses a 64-byte header copied to the host.  Any output may be NULL.
 * stream_bytes is the total container size. */
fmtc_status fmtc_stream_info(const void *h_header, size_t header_bytes, int *bits, int *C, int64_t *P,
                             int *px_per_chunk, int64_t *n_chunks, float *delta, uint64_t *payload_bits,
                             uint64_t *stream_bytes);

/* ---- 8-bit basis, 8-bit activations ----
 * Section 3.1 "Linear transform" stores the PCA matrix at 8 bits; the hardware
 * of section 5 moves 8-bit activations.  Reading taken here, for unsigned
 * 8-bit activations xq with x = act_scale * xq (post-activation maps):
 *   Tq = clamp(rne(T / s_T), -127, 127), s_T = (float)(max|T| / 127);
 *   mf[c] = rne(256 mu[c] / act_scale)   (the mean with 8 fraction bits);
 *   forward: n = 256 sum_c Tq[k][c] xq[c] - sum_c Tq[k][c] mf[c] (exact),
 *            level = clamp(rne(n * g)), g = (s_T act_scale) / (256 Delta) in fp64,
 *            symbol = level + 2^(bits-1);  Delta = fmtc_delta(A of the basis, bits);
 *   inverse: m = sum_k Tq[k][c] (s[k] - 2^(bits-1)) (exact), v = fma(m, h, mf[c]),
 *            h = (s_T Delta 256) / act_scale in fp64, xq^ = clamp(rne(v / 256), 0, 255).
 * Both contractions run on the integer matrix cores and every rounding is one
 * fp64 operation on exact operands: the results are defined bit for bit.
 * The symbols feed the same coder and container as the fp32 path.
 * fmtc_basis8_create derives the 8-bit basis from an fp32 one (host work plus
 * a device upload; `basis` stays valid and independent).  Export pointers may
 * be NULL (h_Tq: C*C row major, h_mean_fix: C). */
typedef struct fmtc_basis8 fmtc_basis8;
fmtc_status fmtc_basis8_create(const fmtc_basis *basis, float act_scale, fmtc_basis8 **out);
fmtc_status fmtc_basis8_export(const fmtc_basis8 *basis, int8_t *h_Tq, float *scale_T, int32_t *h_mean_fix,
                               float *act_scale, float *range_A);
void fmtc_basis8_destroy(fmtc_basis8 *basis);
/* Staged: activations (uint8, N*C*H*W in `layout`, 16-byte aligned) -> symbols
 * [P][C] (16-byte aligned), and symbols -> activations.  Asynchronous. */
fmtc_status fmtc_quantize_u8(const fmtc_basis8 *basis, const uint8_t *d_xq, int64_t N, int C, int H, int W,
                             fmtc_layout layout, int bits, uint8_t *d_syms, void *hip_stream);
fmtc_status fmtc_reconstruct_u8(const fmtc_basis8 *basis, const uint8_t *d_syms, int64_t N, int C, int H, int W,
                                fmtc_layout layout, int bits, uint8_t *d_xq_hat, void *hip_stream);
/* Whole encoder / decoder on 8-bit activations: fmtc_quantize_u8 followed by
 * the coder of fmtc_code_symbols (same stream, bound and workspace size as
 * fmtc_encode), and the decoder: up to 128 channels one kernel (variable length
 * decoding and the integer reconstruction; d_workspace may be NULL), beyond that
 * fmtc_decode_symbols followed by fmtc_reconstruct_u8 with the symbols in
 * d_workspace (at least P*C bytes, 16-byte aligned).
 * Errors and *d_err_flag as for fmtc_encode / fmtc_decode. */
fmtc_status fmtc_encode_u8(const fmtc_basis8 *basis, const uint8_t *d_xq, int64_t N, int C, int H, int W,
                           fmtc_layout layout, int bits, int chunk_syms, void *d_stream_out, size_t cap,
                           uint64_t *d_out_bytes, void *d_workspace, size_t ws_bytes, void *hip_stream);
fmtc_status fmtc_decode_u8(const fmtc_basis8 *basis, const void *d_stream_in, size_t bytes, uint8_t *d_xq_hat,
                           int64_t N, int C, int H, int W, fmtc_layout layout, int bits, uint32_t *d_err_flag,
                           void *d_workspace, size_t ws_bytes, void *hip_stream);

/* ---- instrumentation (not part of the method) ----
 * fmtc_profile_enable(n > 0) creates n HIP event pairs per kernel; from then on
 * every kernel launch of the library carries a pair attached to its own
 * dispatch (start and end of that kernel on the GPU), up to n launches per
 * kernel.  fmtc_profile_enable(0) turns it off and frees the events.
 * fmtc_profile_read waits for the recorded launches of one kernel (index <
 * fmtc_profile_kernels()) and returns their average and minimum duration in
 * milliseconds.  fmtc_profile_copy launches a plain device-to-device copy of
 * `bytes` (a multiple of 16, 16-byte aligned pointers): the known traffic the
 * hardware memory counters are scaled with.  Process-wide, not thread safe. */
fmtc_status fmtc_profile_enable(int max_launches_per_kernel);
int fmtc_profile_kernels(void);
const char *fmtc_profile_name(int kernel);
fmtc_status fmtc_profile_read(int kernel, double *avg_ms, double *min_ms, int *launches);
fmtc_status fmtc_profile_copy(void *d_dst, const void *d_src, size_t bytes, void *hip_stream);

/* Test support (not part of the method): forces one of two equivalent paths so
 * that a test can compare them.  option 0, value 1: fmtc_encode_static always
 * runs projection and packing as two kernels; option 1, value 1: the decoder of
 * wide tensors walks all channel groups of a tile in one workgroup.  Value 0
 * restores the library's own choice.  Process-wide. */
fmtc_status fmtc_test_option(int option, int value);

/* Text of the last error on the calling thread ("" if none). */
const char *fmtc_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* FMTC_H */
