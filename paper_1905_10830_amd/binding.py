"""ctypes binding of libfmtc.so: argument marshalling only.

Every function has the name of the C entry point without the `fmtc_` prefix
and passes torch device tensors as raw pointers on torch's current HIP
stream.  There is no CPU path: if the library is missing or has not been
built the first call raises.
"""
import ctypes
import os

NCHW, NHWC = 0, 1
OK, EINVAL, EBUFSIZE, ECORRUPT, ENOMEM, EHIP = range(6)
ERR_HEADER, ERR_TABLE, ERR_OFFSETS, ERR_CODE = 1, 2, 4, 8

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfmtc.so")

EXPORTS = [
    "fmtc_fit_basis", "fmtc_basis_import", "fmtc_basis_export", "fmtc_basis_channels", "fmtc_basis_destroy",
    "fmtc_delta", "fmtc_encode_bound", "fmtc_workspace_size", "fmtc_encode", "fmtc_encode_noalloc", "fmtc_decode",
    "fmtc_quantize",
    "fmtc_code_symbols", "fmtc_decode_symbols", "fmtc_stream_info", "fmtc_last_error",
    "fmtc_fit_table", "fmtc_table_import", "fmtc_table_export", "fmtc_table_destroy", "fmtc_encode_static_bound",
    "fmtc_encode_static", "fmtc_decode_static",
    "fmtc_fit_state_create", "fmtc_fit_state_update", "fmtc_fit_state_basis", "fmtc_fit_state_count",
    "fmtc_fit_state_destroy", "fmtc_basis_truncate",
    "fmtc_basis8_create", "fmtc_basis8_export", "fmtc_basis8_destroy", "fmtc_quantize_u8", "fmtc_reconstruct_u8",
    "fmtc_encode_u8", "fmtc_decode_u8",
    "fmtc_profile_enable", "fmtc_profile_kernels", "fmtc_profile_name", "fmtc_profile_read", "fmtc_profile_copy",
    "fmtc_test_option",
]

_lib = None


class FmtcError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"fmtc status {status}: {message}")
        self.status = status


def load_library():
    """Loads libfmtc.so (built by paper_1905_10830_amd.build).  Raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} not found: build it with `python -m paper_1905_10830_amd.build` "
            "(there is no fallback implementation)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64, i32, sz, f32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t, ctypes.c_float
    lib.fmtc_fit_basis.argtypes = [vp, i64, i32, i32, i32, i32, vp, ctypes.POINTER(vp)]
    lib.fmtc_basis_import.argtypes = [i32, vp, vp, f32, ctypes.POINTER(vp)]
    lib.fmtc_basis_export.argtypes = [vp, vp, vp, vp, ctypes.POINTER(f32)]
    lib.fmtc_basis_channels.argtypes = [vp]
    lib.fmtc_basis_destroy.argtypes = [vp]
    lib.fmtc_basis_destroy.restype = None
    lib.fmtc_fit_state_create.argtypes = [i32, ctypes.POINTER(vp)]
    lib.fmtc_fit_state_update.argtypes = [vp, vp, i64, i32, i32, i32, i32, vp]
    lib.fmtc_fit_state_basis.argtypes = [vp, vp, i64, i32, i32, i32, i32, vp, ctypes.POINTER(vp)]
    lib.fmtc_fit_state_count.argtypes = [vp]
    lib.fmtc_fit_state_count.restype = i64
    lib.fmtc_fit_state_destroy.argtypes = [vp]
    lib.fmtc_fit_state_destroy.restype = None
    lib.fmtc_basis_truncate.argtypes = [vp, i32, ctypes.POINTER(vp)]
    lib.fmtc_basis8_create.argtypes = [vp, f32, ctypes.POINTER(vp)]
    lib.fmtc_basis8_export.argtypes = [vp, vp, ctypes.POINTER(f32), vp, ctypes.POINTER(f32), ctypes.POINTER(f32)]
    lib.fmtc_basis8_destroy.argtypes = [vp]
    lib.fmtc_basis8_destroy.restype = None
    lib.fmtc_quantize_u8.argtypes = [vp, vp, i64, i32, i32, i32, i32, i32, vp, vp]
    lib.fmtc_reconstruct_u8.argtypes = [vp, vp, i64, i32, i32, i32, i32, i32, vp, vp]
    lib.fmtc_encode_u8.argtypes = [vp, vp, i64, i32, i32, i32, i32, i32, i32, vp, sz, vp, vp, sz, vp]
    lib.fmtc_decode_u8.argtypes = [vp, vp, sz, vp, i64, i32, i32, i32, i32, i32, vp, vp, sz, vp]
    lib.fmtc_delta.argtypes = [f32, i32]
    lib.fmtc_delta.restype = f32
    lib.fmtc_encode_bound.argtypes = [i64, i32, i32, i32]
    lib.fmtc_encode_bound.restype = sz
    lib.fmtc_workspace_size.argtypes = [i64, i32, i32, i32]
    lib.fmtc_workspace_size.restype = sz
    lib.fmtc_encode.argtypes = [vp, vp, i64, i32, i32, i32, i32, i32, i32, vp, sz, vp, vp, sz, vp]
    lib.fmtc_encode_noalloc.argtypes = [vp, vp, i64, i32, i32, i32, i32, i32, i32, vp, sz, vp, vp]
    lib.fmtc_decode.argtypes = [vp, vp, sz, vp, i64, i32, i32, i32, i32, i32, vp, vp]
    lib.fmtc_fit_table.argtypes = [vp, vp, i64, i32, i32, i32, i32, i32, vp, ctypes.POINTER(vp)]
    lib.fmtc_table_import.argtypes = [vp, i32, ctypes.POINTER(vp)]
    lib.fmtc_table_export.argtypes = [vp, vp, ctypes.POINTER(i32)]
    lib.fmtc_table_destroy.argtypes = [vp]
    lib.fmtc_table_destroy.restype = None
    lib.fmtc_encode_static_bound.argtypes = [vp, i64, i32, i32]
    lib.fmtc_encode_static_bound.restype = sz
    lib.fmtc_encode_static.argtypes = [vp, vp, vp, i64, i32, i32, i32, i32, i32, vp, sz, vp, vp, sz, vp]
    lib.fmtc_decode_static.argtypes = [vp, vp, vp, sz, vp, i64, i32, i32, i32, i32, vp, vp]
    lib.fmtc_quantize.argtypes = [vp, vp, i64, i32, i32, i32, i32, i32, vp, vp, vp, sz, vp]
    lib.fmtc_code_symbols.argtypes = [vp, i64, i32, i32, i32, f32, vp, sz, vp, vp, sz, vp]
    lib.fmtc_decode_symbols.argtypes = [vp, sz, i64, i32, i32, vp, vp, vp]
    lib.fmtc_stream_info.argtypes = [vp, sz, ctypes.POINTER(i32), ctypes.POINTER(i32), ctypes.POINTER(i64),
                                     ctypes.POINTER(i32), ctypes.POINTER(i64), ctypes.POINTER(f32),
                                     ctypes.POINTER(ctypes.c_uint64), ctypes.POINTER(ctypes.c_uint64)]
    lib.fmtc_last_error.restype = ctypes.c_char_p
    lib.fmtc_profile_enable.argtypes = [i32]
    lib.fmtc_profile_name.argtypes = [i32]
    lib.fmtc_profile_name.restype = ctypes.c_char_p
    lib.fmtc_profile_read.argtypes = [i32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double),
                                      ctypes.POINTER(i32)]
    lib.fmtc_profile_copy.argtypes = [vp, vp, sz, vp]
    lib.fmtc_test_option.argtypes = [i32, i32]
    _lib = lib
    return lib


def _check(status):
    if status != OK:
        raise FmtcError(status, load_library().fmtc_last_error().decode())


def _stream():
    import torch

    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dims(x, layout):
    if x.dim() != 4:
        raise ValueError("expected a 4-d tensor")
    if layout == NHWC:
        n, h, w, c = x.shape
    else:
        n, c, h, w = x.shape
    return n, c, h, w


def _dev(t, dtype):
    import torch

    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous() and t.dtype == dtype):
        raise ValueError(f"expected a contiguous device tensor of {dtype}")
    return ctypes.c_void_p(t.data_ptr())


class Basis:
    """Owns an fmtc_basis handle."""

    def __init__(self, handle):
        self._h = handle

    @property
    def C(self):
        return load_library().fmtc_basis_channels(self._h)

    def export(self):
        """-> T (C,C) fp32, mu (C) fp32, eigenvalues (C) fp64, range A (numpy / float)."""
        import numpy as np

        c = self.C
        T = np.empty((c, c), np.float32)
        mu = np.empty(c, np.float32)
        eig = np.empty(c, np.float64)
        A = ctypes.c_float(0)
        _check(load_library().fmtc_basis_export(self._h, T.ctypes.data, mu.ctypes.data, eig.ctypes.data,
                                                ctypes.byref(A)))
        return T, mu, eig, np.float32(A.value)

    def truncate(self, keep):
        """-> a new Basis that keeps the `keep` leading components (the other rows of T are zero)."""
        out = ctypes.c_void_p()
        _check(load_library().fmtc_basis_truncate(self._h, int(keep), ctypes.byref(out)))
        return Basis(out)

    def close(self):
        if self._h:
            load_library().fmtc_basis_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def fit_basis(x, layout=NHWC):
    import torch

    n, c, h, w = _dims(x, layout)
    out = ctypes.c_void_p()
    _check(load_library().fmtc_fit_basis(_dev(x, torch.float32), n, c, h, w, layout, _stream(), ctypes.byref(out)))
    return Basis(out)


class Basis8:
    """Owns an fmtc_basis8 handle: the 8-bit basis for unsigned 8-bit activations x = act_scale * xq."""

    def __init__(self, basis, act_scale):
        self._h = ctypes.c_void_p()
        _check(load_library().fmtc_basis8_create(basis._h, float(act_scale), ctypes.byref(self._h)))
        self.C = basis.C

    def export(self):
        """-> Tq int8 (C,C), s_T, mean_fix int32 (C), act_scale, range A."""
        import numpy as np

        Tq = np.empty((self.C, self.C), np.int8)
        mf = np.empty(self.C, np.int32)
        sT, sx, A = ctypes.c_float(0), ctypes.c_float(0), ctypes.c_float(0)
        _check(load_library().fmtc_basis8_export(self._h, Tq.ctypes.data, ctypes.byref(sT), mf.ctypes.data,
                                                 ctypes.byref(sx), ctypes.byref(A)))
        return Tq, np.float32(sT.value), mf, np.float32(sx.value), np.float32(A.value)

    def close(self):
        if self._h:
            load_library().fmtc_basis8_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def quantize_u8(basis8, xq, bits, layout=NHWC, syms=None):
    """Asynchronous.  xq: uint8 device tensor (4-d).  -> symbols uint8 [P, C]."""
    import torch

    n, c, h, w = _dims(xq, layout)
    if syms is None:
        syms = torch.empty((n * h * w, c), dtype=torch.uint8, device=xq.device)
    _check(load_library().fmtc_quantize_u8(basis8._h, _dev(xq, torch.uint8), n, c, h, w, layout, bits,
                                           _dev(syms, torch.uint8), _stream()))
    return syms


def reconstruct_u8(basis8, syms, shape, bits, layout=NHWC, out=None):
    """Asynchronous.  symbols [P, C] -> uint8 activations of the 4-d `shape`."""
    import torch

    if out is None:
        out = torch.empty(tuple(shape), dtype=torch.uint8, device=syms.device)
    n, c, h, w = _dims(out, layout)
    _check(load_library().fmtc_reconstruct_u8(basis8._h, _dev(syms, torch.uint8), n, c, h, w, layout, bits,
                                              _dev(out, torch.uint8), _stream()))
    return out


def encode_u8(basis8, xq, bits, layout=NHWC, chunk_syms=4096, stream_out=None, out_bytes=None, workspace=None):
    """Asynchronous.  -> (stream_out uint8 tensor of capacity encode_bound, out_bytes int64[1] device tensor)."""
    import torch

    n, c, h, w = _dims(xq, layout)
    P = n * h * w
    if stream_out is None:
        stream_out = torch.empty(encode_bound(P, c, bits, chunk_syms), dtype=torch.uint8, device=xq.device)
    if out_bytes is None:
        out_bytes = torch.zeros(1, dtype=torch.int64, device=xq.device)
    if workspace is None:
        workspace = torch.empty(workspace_size(P, c, bits, chunk_syms), dtype=torch.uint8, device=xq.device)
    _check(load_library().fmtc_encode_u8(basis8._h, _dev(xq, torch.uint8), n, c, h, w, layout, bits, chunk_syms,
                                         _dev(stream_out, torch.uint8), stream_out.numel(),
                                         ctypes.c_void_p(out_bytes.data_ptr()), _dev(workspace, torch.uint8),
                                         workspace.numel(), _stream()))
    return stream_out, out_bytes


def decode_u8(basis8, stream_in, shape, bits, layout=NHWC, out=None, err_flag=None, nbytes=None, workspace=None):
    """Asynchronous.  -> (uint8 activations of `shape`, err_flag int32[1] device tensor)."""
    import torch

    if out is None:
        out = torch.empty(tuple(shape), dtype=torch.uint8, device=stream_in.device)
    if err_flag is None:
        err_flag = torch.zeros(1, dtype=torch.int32, device=stream_in.device)
    n, c, h, w = _dims(out, layout)
    if workspace is None and c > 128:  # narrower tensors are decoded and reconstructed by one kernel
        workspace = torch.empty(n * h * w * c, dtype=torch.uint8, device=stream_in.device)
    _check(load_library().fmtc_decode_u8(basis8._h, _dev(stream_in, torch.uint8),
                                         stream_in.numel() if nbytes is None else int(nbytes),
                                         _dev(out, torch.uint8), n, c, h, w, layout, bits,
                                         ctypes.c_void_p(err_flag.data_ptr()),
                                         None if workspace is None else _dev(workspace, torch.uint8),
                                         0 if workspace is None else workspace.numel(), _stream()))
    return out, err_flag


class FitState:
    """Owns an fmtc_fit_state handle: calibration statistics accumulated over several tensors."""

    def __init__(self, C):
        self._h = ctypes.c_void_p()
        _check(load_library().fmtc_fit_state_create(int(C), ctypes.byref(self._h)))

    @property
    def count(self):
        return load_library().fmtc_fit_state_count(self._h)

    def update(self, x, layout=NHWC):
        import torch

        n, c, h, w = _dims(x, layout)
        _check(load_library().fmtc_fit_state_update(self._h, _dev(x, torch.float32), n, c, h, w, layout, _stream()))

    def basis(self, x, layout=NHWC):
        """Basis of everything seen so far; the dynamic range is measured on x."""
        import torch

        n, c, h, w = _dims(x, layout)
        out = ctypes.c_void_p()
        _check(load_library().fmtc_fit_state_basis(self._h, _dev(x, torch.float32), n, c, h, w, layout, _stream(),
                                                   ctypes.byref(out)))
        return Basis(out)

    def close(self):
        if self._h:
            load_library().fmtc_fit_state_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def basis_import(T, mu, range_A):
    import numpy as np

    T = np.ascontiguousarray(T, dtype=np.float32)
    mu = np.ascontiguousarray(mu, dtype=np.float32)
    out = ctypes.c_void_p()
    _check(load_library().fmtc_basis_import(T.shape[0], T.ctypes.data, mu.ctypes.data, float(range_A),
                                            ctypes.byref(out)))
    return Basis(out)


def delta(range_A, bits):
    return load_library().fmtc_delta(float(range_A), int(bits))


def encode_bound(P, C, bits, chunk_syms=4096):
    return load_library().fmtc_encode_bound(P, C, bits, chunk_syms)


def workspace_size(P, C, bits, chunk_syms=4096):
    return load_library().fmtc_workspace_size(P, C, bits, chunk_syms)


def encode(basis, x, bits, layout=NHWC, chunk_syms=4096, stream_out=None, out_bytes=None, workspace=None):
    """Asynchronous.  -> (stream_out uint8 tensor of capacity encode_bound, out_bytes int64[1] device tensor)."""
    import torch

    n, c, h, w = _dims(x, layout)
    P = n * h * w
    if stream_out is None:
        stream_out = torch.empty(encode_bound(P, c, bits, chunk_syms), dtype=torch.uint8, device=x.device)
    if out_bytes is None:
        out_bytes = torch.zeros(1, dtype=torch.int64, device=x.device)
    if workspace is None:
        workspace = torch.empty(workspace_size(P, c, bits, chunk_syms), dtype=torch.uint8, device=x.device)
    _check(load_library().fmtc_encode(basis._h, _dev(x, torch.float32), n, c, h, w, layout, bits, chunk_syms,
                                      _dev(stream_out, torch.uint8), stream_out.numel(),
                                      _dev(out_bytes, torch.int64), _dev(workspace, torch.uint8),
                                      workspace.numel(), _stream()))
    return stream_out, out_bytes


NOALLOC_SCRATCH_BYTES = 6 << 20


def encode_noalloc(basis, x, bits, stream_out, out_bytes, layout=NHWC, chunk_syms=4096):
    """Asynchronous.  fmtc_encode with the workspace in the library's own device array; the caller brings the
    outputs (nothing is allocated here either)."""
    import torch

    n, c, h, w = _dims(x, layout)
    _check(load_library().fmtc_encode_noalloc(basis._h, _dev(x, torch.float32), n, c, h, w, layout, bits, chunk_syms,
                                              _dev(stream_out, torch.uint8), stream_out.numel(),
                                              _dev(out_bytes, torch.int64), _stream()))
    return stream_out, out_bytes


class Table:
    """Owns an fmtc_table handle (a code table fixed at calibration time)."""

    def __init__(self, handle):
        self._h = handle

    def export(self):
        """-> (code lengths uint8[2^bits] numpy, bits)."""
        import numpy as np

        ln = np.zeros(256, np.uint8)
        bits = ctypes.c_int32(0)
        _check(load_library().fmtc_table_export(self._h, ln.ctypes.data, ctypes.byref(bits)))
        return ln[: 1 << bits.value].copy(), bits.value

    @property
    def bits(self):
        return self.export()[1]

    def close(self):
        if self._h:
            load_library().fmtc_table_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def fit_table(basis, x, bits, layout=NHWC):
    import torch

    n, c, h, w = _dims(x, layout)
    out = ctypes.c_void_p()
    _check(load_library().fmtc_fit_table(basis._h, _dev(x, torch.float32), n, c, h, w, layout, bits, _stream(),
                                         ctypes.byref(out)))
    return Table(out)


def table_import(lengths, bits):
    import numpy as np

    ln = np.ascontiguousarray(lengths, dtype=np.uint8)
    if ln.size != 1 << bits:
        raise ValueError("one length per symbol of the alphabet")
    out = ctypes.c_void_p()
    _check(load_library().fmtc_table_import(ln.ctypes.data, bits, ctypes.byref(out)))
    return Table(out)


def encode_static_bound(table, P, C, chunk_syms=4096):
    return load_library().fmtc_encode_static_bound(table._h, P, C, chunk_syms)


def encode_static(basis, table, x, layout=NHWC, chunk_syms=4096, stream_out=None, out_bytes=None, workspace=None):
    """Asynchronous.  -> (stream_out uint8 tensor, out_bytes int64[1] device tensor)."""
    import torch

    n, c, h, w = _dims(x, layout)
    P = n * h * w
    bits = table.bits
    if stream_out is None:
        stream_out = torch.empty(encode_static_bound(table, P, c, chunk_syms), dtype=torch.uint8, device=x.device)
    if out_bytes is None:
        out_bytes = torch.zeros(1, dtype=torch.int64, device=x.device)
    if workspace is None:
        workspace = torch.empty(workspace_size(P, c, bits, chunk_syms), dtype=torch.uint8, device=x.device)
    _check(load_library().fmtc_encode_static(basis._h, table._h, _dev(x, torch.float32), n, c, h, w, layout,
                                             chunk_syms, _dev(stream_out, torch.uint8), stream_out.numel(),
                                             _dev(out_bytes, torch.int64), _dev(workspace, torch.uint8),
                                             workspace.numel(), _stream()))
    return stream_out, out_bytes


def decode_static(basis, table, stream_in, shape, layout=NHWC, xhat=None, err_flag=None, nbytes=None):
    """Asynchronous.  -> (xhat fp32 tensor of `shape`, err_flag int32[1] device tensor)."""
    import torch

    if xhat is None:
        xhat = torch.empty(shape, dtype=torch.float32, device=stream_in.device)
    if err_flag is None:
        err_flag = torch.zeros(1, dtype=torch.int32, device=stream_in.device)
    n, c, h, w = _dims(xhat, layout)
    _check(load_library().fmtc_decode_static(basis._h, table._h, _dev(stream_in, torch.uint8),
                                             stream_in.numel() if nbytes is None else nbytes,
                                             _dev(xhat, torch.float32), n, c, h, w, layout,
                                             _dev(err_flag, torch.int32), _stream()))
    return xhat, err_flag


def decode(basis, stream_in, shape, bits, layout=NHWC, xhat=None, err_flag=None, nbytes=None):
    """Asynchronous.  -> (xhat fp32 tensor of `shape`, err_flag int32[1] device tensor).
    A caller-supplied err_flag must be zero on entry: the decoder only ORs bits into it."""
    import torch

    if xhat is None:
        xhat = torch.empty(shape, dtype=torch.float32, device=stream_in.device)
    if err_flag is None:
        err_flag = torch.zeros(1, dtype=torch.int32, device=stream_in.device)
    n, c, h, w = _dims(xhat, layout)
    _check(load_library().fmtc_decode(basis._h, _dev(stream_in, torch.uint8),
                                      stream_in.numel() if nbytes is None else int(nbytes),
                                      _dev(xhat, torch.float32), n, c, h, w, layout, bits,
                                      _dev(err_flag, torch.int32), _stream()))
    return xhat, err_flag


def quantize(basis, x, bits, layout=NHWC, syms=None, hist=None, workspace=None):
    """Asynchronous.  -> (symbols uint8 [P, C], histogram int32 [256])."""
    import torch

    n, c, h, w = _dims(x, layout)
    P = n * h * w
    if syms is None:
        syms = torch.empty((P, c), dtype=torch.uint8, device=x.device)
    if hist is None:
        hist = torch.zeros(256, dtype=torch.int32, device=x.device)
    if workspace is None:
        workspace = torch.empty(workspace_size(P, c, bits, 4096), dtype=torch.uint8, device=x.device)
    _check(load_library().fmtc_quantize(basis._h, _dev(x, torch.float32), n, c, h, w, layout, bits,
                                        _dev(syms, torch.uint8), _dev(hist, torch.int32),
                                        _dev(workspace, torch.uint8), workspace.numel(), _stream()))
    return syms, hist


def code_symbols(syms, C, bits, delta_value, chunk_syms=4096, stream_out=None, out_bytes=None, workspace=None):
    """Asynchronous.  syms: uint8 device tensor with P*C elements.  -> (stream_out, out_bytes)."""
    import torch

    P = syms.numel() // C
    if stream_out is None:
        stream_out = torch.empty(encode_bound(P, C, bits, chunk_syms), dtype=torch.uint8, device=syms.device)
    if out_bytes is None:
        out_bytes = torch.zeros(1, dtype=torch.int64, device=syms.device)
    if workspace is None:
        workspace = torch.empty(workspace_size(P, C, bits, chunk_syms), dtype=torch.uint8, device=syms.device)
    _check(load_library().fmtc_code_symbols(_dev(syms, torch.uint8), P, C, bits, chunk_syms, float(delta_value),
                                            _dev(stream_out, torch.uint8), stream_out.numel(),
                                            _dev(out_bytes, torch.int64), _dev(workspace, torch.uint8),
                                            workspace.numel(), _stream()))
    return stream_out, out_bytes


def decode_symbols(stream_in, P, C, bits, syms=None, err_flag=None, nbytes=None):
    """Asynchronous.  -> (symbols uint8 [P, C], err_flag int32[1])."""
    import torch

    if syms is None:
        syms = torch.empty((P, C), dtype=torch.uint8, device=stream_in.device)
    if err_flag is None:
        err_flag = torch.zeros(1, dtype=torch.int32, device=stream_in.device)
    _check(load_library().fmtc_decode_symbols(_dev(stream_in, torch.uint8),
                                              stream_in.numel() if nbytes is None else int(nbytes), P, C, bits,
                                              _dev(syms, torch.uint8), _dev(err_flag, torch.int32), _stream()))
    return syms, err_flag


def stream_info(header_bytes):
    """header_bytes: the first 64 bytes of a stream on the host (bytes / numpy uint8)."""
    buf = bytes(bytearray(header_bytes))[:64]
    bits, C, ppc = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    P, nch = ctypes.c_int64(), ctypes.c_int64()
    dlt = ctypes.c_float()
    pbits, sbytes = ctypes.c_uint64(), ctypes.c_uint64()
    _check(load_library().fmtc_stream_info(buf, len(buf), ctypes.byref(bits), ctypes.byref(C), ctypes.byref(P),
                                           ctypes.byref(ppc), ctypes.byref(nch), ctypes.byref(dlt),
                                           ctypes.byref(pbits), ctypes.byref(sbytes)))
    return dict(bits=bits.value, C=C.value, P=P.value, px_per_chunk=ppc.value, n_chunks=nch.value,
                delta=dlt.value, payload_bits=pbits.value, stream_bytes=sbytes.value)


TEST_STATIC_TWO_KERNELS, TEST_DECODE_ONE_ROW = 0, 1


def test_option(option, value):
    """Forces one of two equivalent paths (tests only); value 0 restores the library's own choice."""
    _check(load_library().fmtc_test_option(int(option), int(value)))


test_option.__test__ = False  # (not a test, whatever a collector makes of the name)


def profile_enable(max_launches_per_kernel):
    _check(load_library().fmtc_profile_enable(int(max_launches_per_kernel)))


def profile_copy(dst, src):
    """Yardstick copy of src into dst (uint8 device tensors of equal size, a multiple of 16 bytes)."""
    import torch

    _check(load_library().fmtc_profile_copy(_dev(dst, torch.uint8), _dev(src, torch.uint8), src.numel(), _stream()))


def profile_read():
    """-> {kernel name: (avg_ms, min_ms, launches)} for the kernels launched since profile_enable."""
    lib = load_library()
    out = {}
    for k in range(lib.fmtc_profile_kernels()):
        avg, mn, n = ctypes.c_double(), ctypes.c_double(), ctypes.c_int()
        _check(lib.fmtc_profile_read(k, ctypes.byref(avg), ctypes.byref(mn), ctypes.byref(n)))
        if n.value:
            out[lib.fmtc_profile_name(k).decode()] = (avg.value, mn.value, n.value)
    return out
