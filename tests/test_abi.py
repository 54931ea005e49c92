"""CPU-side checks of the C-ABI library: it loads, exports every declared entry
point, and its host-only helpers agree with the oracle's container geometry."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_1905_10830_amd import binding as fmtc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(fmtc.LIB_PATH):
        from paper_1905_10830_amd import build

        build.build()
    return fmtc.load_library()


def _declared():
    text = open(os.path.join(ROOT, "include", "fmtc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fmtc_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared()
    assert sorted(names) == sorted(fmtc.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_no_torch_types_in_the_header():
    text = open(os.path.join(ROOT, "include", "fmtc.h")).read()
    assert "at::" not in text and "torch" not in text.lower().replace("pytorch", "")
    assert 'extern "C"' in text


def test_delta_matches_oracle(lib, oracle):
    for A in (0.0, 1.0, 3.7, 127.0, 1e-3, 55.5):
        for bits in range(2, 9):
            assert np.float32(fmtc.delta(A, bits)) == oracle.delta(A, bits)


def test_sizes_match_oracle_geometry(lib, oracle):
    for P, C, bits, cs in [(3136, 64, 8, 4096), (25088, 128, 6, 4096), (200704, 144, 5, 4096), (3136, 960, 5, 4096),
                           (77, 3, 3, 64), (1, 1, 2, 64), (1000, 50, 4, 4096)]:
        assert fmtc.encode_bound(P, C, bits, cs) == oracle.stream_bound(P, C, bits, cs)
        assert fmtc.workspace_size(P, C, bits, cs) >= P * C
    assert fmtc.encode_bound(0, 64, 4, 4096) == 0
    assert fmtc.encode_bound(10, 2000, 4, 4096) == 0
    assert fmtc.encode_bound(10, 64, 9, 4096) == 0
    assert fmtc.encode_bound(1 << 40, 64, 4, 4096) == 0  # V must stay below 2^32


def test_stream_info_parses_an_oracle_header(lib, oracle):
    rng = np.random.default_rng(0)
    sym = rng.integers(0, 16, (500, 24)).astype(np.uint8)
    h = oracle.histogram(sym, 4)
    ln = oracle.huffman_lengths(h[:16])
    stream = oracle.pack(sym, 24, 4, 0.375, ln, oracle.canonical_codes(ln))
    info = fmtc.stream_info(stream[:64])
    ref = oracle.parse_header(stream)
    assert info["bits"] == 4 and info["C"] == 24 and info["P"] == 500
    assert info["px_per_chunk"] == ref["px_per_chunk"] and info["n_chunks"] == ref["n_chunks"]
    assert info["delta"] == 0.375 and info["payload_bits"] == ref["payload_bits"]
    assert info["stream_bytes"] == len(stream)
    bad = stream[:64].copy()
    bad[0] ^= 1
    with pytest.raises(fmtc.FmtcError) as e:
        fmtc.stream_info(bad)
    assert e.value.status == fmtc.ECORRUPT


def test_argument_errors_are_reported_on_the_host(lib):
    """NULL / range errors come back as a status before anything is launched."""
    out = ctypes.c_void_p()
    st = lib.fmtc_basis_import(0, None, None, 1.0, ctypes.byref(out))
    assert st == fmtc.EINVAL and b"basis" in lib.fmtc_last_error()
    st = lib.fmtc_encode(None, None, 1, 64, 8, 8, fmtc.NHWC, 4, 4096, None, 0, None, None, 0, None)
    assert st == fmtc.EINVAL
    st = lib.fmtc_decode(None, None, 0, None, 1, 64, 8, 8, fmtc.NHWC, 4, None, None)
    assert st == fmtc.EINVAL
    st = lib.fmtc_decode_symbols(None, 0, 10, 64, 4, None, None, None)
    assert st == fmtc.EINVAL


def test_fixed_table_argument_errors_are_reported_on_the_host(lib):
    """The lengths of an imported table are checked before any device memory is touched."""
    out = ctypes.c_void_p()
    flat = (ctypes.c_uint8 * 16)(*([3] * 16))                    # Kraft sum 2: not a prefix code
    assert lib.fmtc_table_import(flat, 4, ctypes.byref(out)) == fmtc.EINVAL
    assert b"prefix code" in lib.fmtc_last_error()
    short = (ctypes.c_uint8 * 16)(*([5] * 16))                   # Kraft sum 1/2: not complete
    assert lib.fmtc_table_import(short, 4, ctypes.byref(out)) == fmtc.EINVAL
    missing = (ctypes.c_uint8 * 16)(*([1] + [0] * 15))           # a symbol without a code
    assert lib.fmtc_table_import(missing, 4, ctypes.byref(out)) == fmtc.EINVAL
    good = (ctypes.c_uint8 * 16)(*([4] * 16))
    assert lib.fmtc_table_import(good, 9, ctypes.byref(out)) == fmtc.EINVAL   # bit depth out of range
    assert lib.fmtc_table_import(None, 4, ctypes.byref(out)) == fmtc.EINVAL
    assert lib.fmtc_encode_static_bound(None, 100, 64, 4096) == 0
    st = lib.fmtc_encode_static(None, None, None, 1, 64, 8, 8, fmtc.NHWC, 4096, None, 0, None, None, 0, None)
    assert st == fmtc.EINVAL
    st = lib.fmtc_decode_static(None, None, None, 0, None, 1, 64, 8, 8, fmtc.NHWC, None, None)
    assert st == fmtc.EINVAL
    st = lib.fmtc_fit_table(None, None, 1, 64, 8, 8, fmtc.NHWC, 4, None, ctypes.byref(out))
    assert st == fmtc.EINVAL
    lib.fmtc_table_destroy(None)  # a no-op


def test_fit_state_and_truncation_argument_errors_are_reported_on_the_host(lib):
    """A fit state lives on the host; its argument checks and those of the truncation need no GPU."""
    st = ctypes.c_void_p()
    assert lib.fmtc_fit_state_create(0, ctypes.byref(st)) == fmtc.EINVAL
    assert lib.fmtc_fit_state_create(2000, ctypes.byref(st)) == fmtc.EINVAL
    assert lib.fmtc_fit_state_create(16, None) == fmtc.EINVAL
    assert lib.fmtc_fit_state_create(16, ctypes.byref(st)) == fmtc.OK and st.value
    assert lib.fmtc_fit_state_count(st) == 0
    assert lib.fmtc_fit_state_count(None) == 0
    assert lib.fmtc_fit_state_update(st, None, 1, 16, 4, 4, fmtc.NHWC, None) == fmtc.EINVAL
    assert lib.fmtc_fit_state_update(None, None, 1, 16, 4, 4, fmtc.NHWC, None) == fmtc.EINVAL
    out = ctypes.c_void_p()
    assert lib.fmtc_fit_state_basis(st, None, 1, 16, 4, 4, fmtc.NHWC, None, ctypes.byref(out)) == fmtc.EINVAL
    assert lib.fmtc_fit_state_basis(st, None, 1, 16, 4, 4, fmtc.NHWC, None, None) == fmtc.EINVAL
    lib.fmtc_fit_state_destroy(st)
    lib.fmtc_fit_state_destroy(None)  # a no-op
    assert lib.fmtc_basis_truncate(None, 4, ctypes.byref(out)) == fmtc.EINVAL
    assert lib.fmtc_basis_truncate(None, 4, None) == fmtc.EINVAL


def test_u8_argument_errors_are_reported_on_the_host(lib):
    out = ctypes.c_void_p()
    assert lib.fmtc_basis8_create(None, 0.5, ctypes.byref(out)) == fmtc.EINVAL
    assert lib.fmtc_basis8_create(None, 0.5, None) == fmtc.EINVAL
    assert lib.fmtc_quantize_u8(None, None, 1, 16, 4, 4, fmtc.NHWC, 6, None, None) == fmtc.EINVAL
    assert lib.fmtc_reconstruct_u8(None, None, 1, 16, 4, 4, fmtc.NHWC, 6, None, None) == fmtc.EINVAL
    assert lib.fmtc_encode_u8(None, None, 1, 16, 4, 4, fmtc.NHWC, 6, 4096, None, 0, None, None, 0, None) == fmtc.EINVAL
    assert lib.fmtc_decode_u8(None, None, 0, None, 1, 16, 4, 4, fmtc.NHWC, 6, None, None, 0, None) == fmtc.EINVAL
    lib.fmtc_basis8_destroy(None)  # a no-op


def test_bench_refuses_more_than_one_gpu():
    """The benchmark is a one-GPU measurement: any other count ends with a message, before anything touches a GPU."""
    import subprocess
    import sys

    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one-GPU" in r.stderr and "--gpus 1" in r.stderr
