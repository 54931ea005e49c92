"""ctypes front end of the fp64 CPU oracle (oracle/fmtc_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the
benchmark's cpu_baseline leg.  It never imports the GPU package and the GPU
package never imports it.  Marshalling only; every step of the method is in C.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fmtc_oracle.c")
_LIB = os.path.join(_HERE, "libfmtc_oracle.so")

NCHW, NHWC = 0, 1
OK, EINVAL, EBUFSIZE, ECORRUPT, ENOMEM = 0, 1, 2, 3, 4


def build(force=False):
    """Compile the oracle with gcc (plain C11, -O2, no vector or threading flags)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.run(
            ["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"],
            check=True,
        )
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.fmtc_oracle_delta.restype = ctypes.c_float
        _lib.fmtc_oracle_delta.argtypes = [ctypes.c_float, ctypes.c_int]
        _lib.fmtc_oracle_entropy.restype = ctypes.c_double
        _lib.fmtc_oracle_mse.restype = ctypes.c_double
        _lib.fmtc_oracle_stream_bound.restype = ctypes.c_size_t
    return _lib


class OracleError(RuntimeError):
    def __init__(self, code, what):
        super().__init__(f"{what}: oracle status {code}")
        self.code = code


def _chk(code, what):
    if code != OK:
        raise OracleError(code, what)


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _dims(x, layout):
    """Logical (N, C, HW) of a 4-d array stored in the given layout."""
    if x.ndim != 4:
        raise ValueError("expected a 4-d tensor")
    if layout == NHWC:
        n, h, w, c = x.shape
    else:
        n, c, h, w = x.shape
    return n, c, h * w


def covariance(x, layout=NHWC):
    x = _f32(x)
    n, c, hw = _dims(x, layout)
    mean = np.empty(c, np.float64)
    cov = np.empty((c, c), np.float64)
    _chk(lib().fmtc_oracle_covariance(_p(x), ctypes.c_int64(n), c, ctypes.c_int64(hw), layout, _p(mean), _p(cov)),
         "covariance")
    return mean, cov


def pca(cov):
    cov = np.ascontiguousarray(cov, dtype=np.float64)
    c = cov.shape[0]
    T = np.empty((c, c), np.float64)
    eig = np.empty(c, np.float64)
    _chk(lib().fmtc_oracle_pca(_p(cov), c, _p(T), _p(eig)), "pca")
    return T, eig


def fit(x, layout=NHWC):
    """-> T (fp32 CxC, rows = components), mu (fp32 C), eigenvalues (fp64), range A (fp32)."""
    x = _f32(x)
    n, c, hw = _dims(x, layout)
    T = np.empty((c, c), np.float32)
    mu = np.empty(c, np.float32)
    eig = np.empty(c, np.float64)
    A = ctypes.c_float(0)
    _chk(lib().fmtc_oracle_fit(_p(x), ctypes.c_int64(n), c, ctypes.c_int64(hw), layout, _p(T), _p(mu), _p(eig),
                               ctypes.byref(A)), "fit")
    return T, mu, eig, np.float32(A.value)


def dynamic_range(x, t0, mu, layout=NHWC):
    """A = max |t0 . (x - mu)| over the pixels of x (fp32 row and mean)."""
    x, t0, mu = _f32(x), _f32(t0), _f32(mu)
    n, c, hw = _dims(x, layout)
    A = ctypes.c_float(0)
    _chk(lib().fmtc_oracle_range(_p(x), ctypes.c_int64(n), c, ctypes.c_int64(hw), layout, _p(t0), _p(mu),
                                 ctypes.byref(A)), "range")
    return np.float32(A.value)


def _pixel_major(x, layout):
    """The tensor's values as [P, C] in logical (n, h, w) pixel order: a copy, no arithmetic."""
    x = _f32(x)
    if layout == NCHW:
        x = np.transpose(x, (0, 2, 3, 1))
    return np.ascontiguousarray(x).reshape(-1, x.shape[-1])


def fit_online(batches, range_x, layout=NHWC):
    """Calibration over several tensors: the fit of their concatenation (mean, covariance, PCA, fp32
    rounding), with the dynamic range measured on range_x.  -> T, mu, eigenvalues, A."""
    allpx = np.concatenate([_pixel_major(b, layout) for b in batches], axis=0)
    mean, cov = covariance(allpx.reshape(1, allpx.shape[0], 1, allpx.shape[1]), NHWC)
    Td, eig = pca(cov)
    T, mu = Td.astype(np.float32), mean.astype(np.float32)
    return T, mu, eig, dynamic_range(range_x, T[0], mu, layout)


def project_keep(x, T, mu, keep, layout=NHWC):
    """Projection onto the `keep` leading components; dropped coefficients are 0.  -> y fp64 [P, C]."""
    x, T, mu = _f32(x), _f32(T), _f32(mu)
    n, c, hw = _dims(x, layout)
    y = np.empty((n * hw, c), np.float64)
    _chk(lib().fmtc_oracle_project_keep(_p(x), ctypes.c_int64(n), c, ctypes.c_int64(hw), layout, _p(T), _p(mu),
                                        int(keep), _p(y)), "project_keep")
    return y


def reconstruct_keep(sym, shape, T, mu, dlt, bits, keep, layout=NHWC):
    """symbols [P, C] -> x_hat fp64 from the `keep` leading components only."""
    sym = np.ascontiguousarray(sym, dtype=np.uint8)
    T, mu = _f32(T), _f32(mu)
    xhat = np.empty(shape, np.float64)
    n, c, hw = _dims(xhat, layout)
    _chk(lib().fmtc_oracle_reconstruct_keep(_p(sym), ctypes.c_int64(n), c, ctypes.c_int64(hw), layout, int(bits),
                                            ctypes.c_float(float(dlt)), _p(T), _p(mu), int(keep), _p(xhat)),
         "reconstruct_keep")
    return xhat


def encode_keep(x, T, mu, dlt, bits, keep, layout=NHWC, chunk_syms=4096, want_margin=False):
    """Encoder with truncation: project_keep, quantizer, this tensor's Huffman table, container."""
    y = project_keep(x, T, mu, keep, layout)
    q = quantize(y, dlt, bits, want_margin)
    sym, margin = q if want_margin else (q, None)
    hist = histogram(sym, bits)
    length = huffman_lengths(hist[: 1 << bits])
    res = {"stream": pack(sym, sym.shape[1], bits, dlt, length, canonical_codes(length), chunk_syms),
           "sym": sym, "hist": hist}
    if want_margin:
        res["margin"] = margin
    return res


def basis8(T, mu, act_scale):
    """8-bit basis for 8-bit activations.  -> Tq int8 [C, C], s_T fp32, mean_fix int32 [C]."""
    T, mu = _f32(T), _f32(mu)
    c = T.shape[0]
    Tq = np.empty((c, c), np.int8)
    mf = np.empty(c, np.int32)
    sT = ctypes.c_float(0)
    _chk(lib().fmtc_oracle_basis8(_p(T), _p(mu), c, ctypes.c_float(float(act_scale)), _p(Tq), ctypes.byref(sT),
                                  _p(mf)), "basis8")
    return Tq, np.float32(sT.value), mf


def quantize_u8(xq, Tq, scale_T, mean_fix, act_scale, dlt, bits, layout=NHWC):
    """uint8 activations (4-d, given layout) -> symbols [P, C] under the 8-bit basis."""
    xq = np.ascontiguousarray(xq, dtype=np.uint8)
    Tq = np.ascontiguousarray(Tq, dtype=np.int8)
    mf = np.ascontiguousarray(mean_fix, dtype=np.int32)
    n, c, hw = _dims(xq, layout)
    sym = np.empty((n * hw, c), np.uint8)
    _chk(lib().fmtc_oracle_quantize_u8(_p(xq), ctypes.c_int64(n), c, ctypes.c_int64(hw), layout, _p(Tq),
                                       ctypes.c_float(float(scale_T)), _p(mf), ctypes.c_float(float(act_scale)),
                                       ctypes.c_float(float(dlt)), int(bits), _p(sym)), "quantize_u8")
    return sym


def reconstruct_u8(sym, shape, Tq, scale_T, mean_fix, act_scale, dlt, bits, layout=NHWC):
    """symbols [P, C] -> uint8 activations of the given 4-d storage shape."""
    sym = np.ascontiguousarray(sym, dtype=np.uint8)
    Tq = np.ascontiguousarray(Tq, dtype=np.int8)
    mf = np.ascontiguousarray(mean_fix, dtype=np.int32)
    out = np.empty(shape, np.uint8)
    n, c, hw = _dims(out, layout)
    _chk(lib().fmtc_oracle_reconstruct_u8(_p(sym), ctypes.c_int64(n), c, ctypes.c_int64(hw), layout, _p(Tq),
                                          ctypes.c_float(float(scale_T)), _p(mf),
                                          ctypes.c_float(float(act_scale)), ctypes.c_float(float(dlt)), int(bits),
                                          _p(out)), "reconstruct_u8")
    return out


def delta(range_A, bits):
    return np.float32(lib().fmtc_oracle_delta(ctypes.c_float(float(range_A)), int(bits)))


def project(x, T, mu, layout=NHWC):
    """-> y fp64 [P, C], pixel major / coefficient minor."""
    x, T, mu = _f32(x), _f32(T), _f32(mu)
    n, c, hw = _dims(x, layout)
    y = np.empty((n * hw, c), np.float64)
    _chk(lib().fmtc_oracle_project(_p(x), ctypes.c_int64(n), c, ctypes.c_int64(hw), layout, _p(T), _p(mu), _p(y)),
         "project")
    return y


def quantize(y, dlt, bits, want_margin=False):
    y = np.ascontiguousarray(y, dtype=np.float64)
    sym = np.empty(y.shape, np.uint8)
    margin = np.empty(y.shape, np.float64) if want_margin else None
    _chk(lib().fmtc_oracle_quantize(_p(y), ctypes.c_int64(y.size), ctypes.c_float(float(dlt)), int(bits), _p(sym),
                                    _p(margin) if want_margin else None), "quantize")
    return (sym, margin) if want_margin else sym


def histogram(sym, bits):
    sym = np.ascontiguousarray(sym, dtype=np.uint8)
    hist = np.empty(256, np.uint64)
    _chk(lib().fmtc_oracle_histogram(_p(sym), ctypes.c_int64(sym.size), int(bits), _p(hist)), "histogram")
    return hist


def entropy(hist):
    hist = np.ascontiguousarray(hist, dtype=np.uint64)
    return float(lib().fmtc_oracle_entropy(_p(hist), int(hist.size)))


def huffman_lengths(hist):
    hist = np.ascontiguousarray(hist, dtype=np.uint64)
    length = np.empty(hist.size, np.uint8)
    _chk(lib().fmtc_oracle_huffman_lengths(_p(hist), int(hist.size), _p(length)), "huffman_lengths")
    return length


def static_lengths(calib_hist):
    """Lengths of a code table fixed at calibration time, from the calibration symbols' counts [2^bits]."""
    hist = np.ascontiguousarray(calib_hist, dtype=np.uint64)
    length = np.empty(hist.size, np.uint8)
    _chk(lib().fmtc_oracle_static_lengths(_p(hist), int(hist.size), _p(length)), "static_lengths")
    return length


def canonical_codes(length):
    length = np.ascontiguousarray(length, dtype=np.uint8)
    code = np.empty(length.size, np.uint64)
    _chk(lib().fmtc_oracle_canonical_codes(_p(length), int(length.size), _p(code)), "canonical_codes")
    return code


def stream_bound(P, C, bits, chunk_syms=4096):
    return int(lib().fmtc_oracle_stream_bound(ctypes.c_int64(P), int(C), int(bits), int(chunk_syms)))


def pack(sym, C, bits, dlt, length, code, chunk_syms=4096, cap=None):
    """sym: [P, C] (or flat P*C) symbols -> container bytes (uint8 array)."""
    sym = np.ascontiguousarray(sym, dtype=np.uint8)
    P = sym.size // C
    if cap is None:
        cap = stream_bound(P, C, bits, chunk_syms)
    out = np.zeros(max(cap, 1), np.uint8)
    nbytes = ctypes.c_size_t(0)
    length = np.ascontiguousarray(length, dtype=np.uint8)
    code = np.ascontiguousarray(code, dtype=np.uint64)
    _chk(lib().fmtc_oracle_pack(_p(sym), ctypes.c_int64(P), int(C), int(bits), int(chunk_syms),
                                ctypes.c_float(float(dlt)), _p(length), _p(code), _p(out), ctypes.c_size_t(cap),
                                ctypes.byref(nbytes)), "pack")
    return out[: nbytes.value].copy()


def unpack(stream, P, C, bits):
    """-> symbols [P, C], delta, payload bits."""
    stream = np.ascontiguousarray(stream, dtype=np.uint8)
    sym = np.empty((P, C), np.uint8)
    dlt = ctypes.c_float(0)
    pbits = ctypes.c_uint64(0)
    _chk(lib().fmtc_oracle_unpack(_p(stream), ctypes.c_size_t(stream.size), ctypes.c_int64(P), int(C), int(bits),
                                  _p(sym), ctypes.byref(dlt), ctypes.byref(pbits)), "unpack")
    return sym, np.float32(dlt.value), int(pbits.value)


def reconstruct(sym, shape, T, mu, dlt, bits, layout=NHWC):
    """symbols [P, C] -> x_hat fp64 with the given 4-d storage shape."""
    sym = np.ascontiguousarray(sym, dtype=np.uint8)
    T, mu = _f32(T), _f32(mu)
    xhat = np.empty(shape, np.float64)
    n, c, hw = _dims(xhat, layout)
    _chk(lib().fmtc_oracle_reconstruct(_p(sym), ctypes.c_int64(n), c, ctypes.c_int64(hw), layout, int(bits),
                                       ctypes.c_float(float(dlt)), _p(T), _p(mu), _p(xhat)), "reconstruct")
    return xhat


def mse(x, xhat):
    x = _f32(x)
    xhat = np.ascontiguousarray(xhat, dtype=np.float64)
    return float(lib().fmtc_oracle_mse(_p(x), _p(xhat), ctypes.c_int64(x.size)))


def encode(x, T, mu, dlt, bits, layout=NHWC, chunk_syms=4096, want_margin=False):
    """Whole encoder.  -> dict(stream, sym [P,C], hist, margin?)."""
    x, T, mu = _f32(x), _f32(T), _f32(mu)
    n, c, hw = _dims(x, layout)
    P = n * hw
    cap = stream_bound(P, c, bits, chunk_syms)
    out = np.zeros(cap, np.uint8)
    sym = np.empty((P, c), np.uint8)
    margin = np.empty((P, c), np.float64) if want_margin else None
    hist = np.empty(256, np.uint64)
    nbytes = ctypes.c_size_t(0)
    _chk(lib().fmtc_oracle_encode(_p(x), ctypes.c_int64(n), c, ctypes.c_int64(hw), layout, _p(T), _p(mu),
                                  ctypes.c_float(float(dlt)), int(bits), int(chunk_syms), _p(out),
                                  ctypes.c_size_t(cap), ctypes.byref(nbytes), _p(sym),
                                  _p(margin) if want_margin else None, _p(hist)), "encode")
    res = {"stream": out[: nbytes.value].copy(), "sym": sym, "hist": hist}
    if want_margin:
        res["margin"] = margin
    return res


def encode_static(x, T, mu, dlt, bits, length, layout=NHWC, chunk_syms=4096):
    """Encoder with a given code table (lengths of all 2^bits symbols).  -> dict(stream, sym [P,C])."""
    y = project(x, T, mu, layout)
    sym = quantize(y, dlt, bits)
    length = np.ascontiguousarray(length, dtype=np.uint8)
    cap = stream_bound(sym.shape[0], sym.shape[1], bits, chunk_syms) + sym.size * int(length.max()) // 8
    return {"stream": pack(sym, sym.shape[1], bits, dlt, length, canonical_codes(length), chunk_syms, cap=cap),
            "sym": sym}


def decode(stream, shape, T, mu, bits, layout=NHWC):
    """Whole decoder.  -> x_hat fp64 (storage shape), symbols [P, C]."""
    stream = np.ascontiguousarray(stream, dtype=np.uint8)
    T, mu = _f32(T), _f32(mu)
    xhat = np.empty(shape, np.float64)
    n, c, hw = _dims(xhat, layout)
    sym = np.empty((n * hw, c), np.uint8)
    _chk(lib().fmtc_oracle_decode(_p(stream), ctypes.c_size_t(stream.size), ctypes.c_int64(n), c,
                                  ctypes.c_int64(hw), layout, int(bits), _p(T), _p(mu), _p(xhat), _p(sym)),
         "decode")
    return xhat, sym


def parse_header(stream):
    """Header fields of a container as a dict (byte layout documented in fmtc_oracle.c)."""
    b = np.ascontiguousarray(stream[:64], dtype=np.uint8).tobytes()
    import struct

    magic, version, bits, _r0, C, ppc, P, n_chunks, sub_syms, dlt, spc, pw, pb, _r1 = struct.unpack(
        "<IHBBIIQIIfIQQQ", b)
    return dict(magic=magic, version=version, bits=bits, C=C, px_per_chunk=ppc, P=P, n_chunks=n_chunks,
                sub_syms=sub_syms, delta=dlt, subs_per_chunk=spc, payload_words=pw, payload_bits=pb)
