"""GPU parity at the full sizes of the benchmark configurations, in the launch
configuration bench.py times (NHWC, 4096-symbol chunks, basis fitted on the
8-image calibration batch of the same seed stream).

The C oracle finishes every single-tensor configuration in seconds, so every
output is compared, not a sample: the whole encoder output (symbols per the
boundary rule, stream bytes bit-exact given the symbols) and the whole decoder
output (<= 1e-4 max-abs to the oracle's fp64 reconstruction of the same symbols).
"""
import numpy as np
import pytest

from paper_1905_10830_amd import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

SYM_MARGIN = 1e-4
SYM_RATE = 1e-6
RECON_TOL = 1e-4

# (workload, bits) -- every single-GPU configuration of the benchmark definition, and two shapes of the
# N = 256 sweep at the ends of its bit range
FULL = [
    ("cfg0_c64_56", 8),
    ("resnet18_stage2_c128_28", 6),
    ("resnet18_stage2_c128_28", 4),
    ("resnet18_stage3_c256_14", 4),
    ("resnet18_stage4_c512_7", 4),
    ("mbv2_c144_56", 5),
    ("mbv2_c960_7", 5),
    ("resnet18_n256_c64_56", 8),
    ("resnet18_n256_c64_56", 6),    # the benchmark's headline: the chunk decoder with four wavefronts per SIMD
    ("resnet18_n256_c128_28", 6),   # ... and with three, the lower parts of its basis read from global memory
    ("resnet18_n256_c128_28", 2),
    ("resnet18_n256_c128_28", 8),   # (the 256-bin histograms leave no room for the eight-wavefront projection)
    ("resnet18_n256_c256_14", 4),
    ("resnet18_n256_c512_7", 3),
]


@pytest.fixture(scope="module")
def fmtc():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1905_10830_amd import binding

    binding.load_library()
    return binding


def fit_on_host(oracle, calib, C):
    """Basis for parity: the oracle's own fit where its Jacobi solver is fast enough, else the oracle's
    covariance with the library eigensolver (any orthonormal basis serves codec parity)."""
    if C <= 256:
        T, mu, _, A = oracle.fit(calib)
        return T, mu, A
    mean, cov = oracle.covariance(calib)
    w, v = np.linalg.eigh(cov)
    T = np.ascontiguousarray(v[:, ::-1].T).astype(np.float32)
    mu = mean.astype(np.float32)
    A = np.float32(np.abs(oracle.project(calib, T, mu)[:, 0]).max())
    return T, mu, A


@pytest.mark.parametrize("name,bits", FULL, ids=[f"{n}_b{b}" for n, b in FULL])
def test_full_size_encode_decode(fmtc, oracle, name, bits):
    wl = synth.WORKLOADS[name]
    C = wl["C"]
    calib, x = synth.workload(name, seed=0)
    T, mu, A = fit_on_host(oracle, calib, C)
    del calib
    d = oracle.delta(A, bits)
    P = x.size // C
    print(f"{name} b={bits}: V={x.size}", flush=True)

    basis = fmtc.basis_import(T, mu, A)
    x_d = torch.from_numpy(x).cuda()
    stream, nbytes = fmtc.encode(basis, x_d, bits, synth.NHWC)
    xhat, err = fmtc.decode(basis, stream, x.shape, bits, synth.NHWC)
    torch.cuda.synchronize()
    n = int(nbytes.item())
    got = stream[:n].cpu().numpy()
    xhat = xhat.cpu().numpy()
    assert int(err.item()) == 0
    del x_d, stream

    # ---- the encoder: the GPU container read by the oracle's decoder, symbols against the oracle's quantizer ----
    sym_gpu, d2, pbits = oracle.unpack(got, P, C, bits)
    assert d2 == d
    y = oracle.project(x, T, mu)
    ref_sym, margin = oracle.quantize(y, d, bits, want_margin=True)
    del y
    diff = sym_gpu != ref_sym
    n_bad = int(diff.sum())
    if n_bad:
        assert margin[diff].max() <= SYM_MARGIN, f"{n_bad} symbols differ, worst margin {margin[diff].max():.3e}"
        assert n_bad / ref_sym.size <= SYM_RATE
    del margin, diff
    # the stream is the oracle's coding of the symbols the GPU quantizer produced: histogram, table, offsets,
    # run sizes and payload bit for bit
    h = oracle.histogram(sym_gpu, bits)
    ln = oracle.huffman_lengths(h[: 1 << bits])
    again = oracle.pack(sym_gpu, C, bits, d, ln, oracle.canonical_codes(ln))
    assert len(again) == n and (got == again).all()
    assert pbits == int((h[: 1 << bits] * ln.astype(np.uint64)).sum())

    # ---- the decoder: every reconstructed value against the oracle's fp64 inverse of the same symbols ----
    worst = 0.0
    hw, n_img = wl["H"] * wl["W"], x.shape[0]
    slab = max(1, n_img // 8)  # images per slab: the fp64 reference of the largest tensors is big
    for n0 in range(0, n_img, slab):
        n1 = min(n_img, n0 + slab)
        ref = oracle.reconstruct(sym_gpu[n0 * hw:n1 * hw], x[n0:n1].shape, T, mu, d, bits)
        worst = max(worst, float(np.abs(xhat[n0:n1].astype(np.float64) - ref).max()))
    assert worst <= RECON_TOL, f"reconstruction off by {worst:.3e}"


# the shapes the one-kernel encoder with a fixed table takes, at full size: one chunk group per workgroup
# (stage 2), and many more groups than the device holds workgroups (N = 256)
STATIC = [
    ("resnet18_stage2_c128_28", 6),
    ("cfg0_c64_56", 8),
    ("resnet18_n256_c128_28", 4),
    ("resnet18_n256_c64_56", 6),
]


@pytest.mark.parametrize("name,bits", STATIC, ids=[f"{n}_b{b}" for n, b in STATIC])
def test_full_size_static_table_encode(fmtc, oracle, name, bits):
    wl = synth.WORKLOADS[name]
    C = wl["C"]
    calib, x = synth.workload(name, seed=0)
    T, mu, A = fit_on_host(oracle, calib, C)
    d = oracle.delta(A, bits)
    P = x.size // C
    print(f"{name} b={bits}: V={x.size}", flush=True)
    basis = fmtc.basis_import(T, mu, A)
    table = fmtc.fit_table(basis, torch.from_numpy(calib).cuda(), bits, synth.NHWC)
    ln, _ = table.export()
    x_d = torch.from_numpy(x).cuda()
    stream, nbytes = fmtc.encode_static(basis, table, x_d, synth.NHWC)
    xhat, err = fmtc.decode(basis, stream, x.shape, bits, synth.NHWC)
    torch.cuda.synchronize()
    n = int(nbytes.item())
    got = stream[:n].cpu().numpy()
    assert int(err.item()) == 0
    sym_gpu, d2, pbits = oracle.unpack(got, P, C, bits)
    assert d2 == d
    ref_sym, margin = oracle.quantize(oracle.project(x, T, mu), d, bits, want_margin=True)
    diff = sym_gpu != ref_sym
    n_bad = int(diff.sum())
    if n_bad:
        assert margin[diff].max() <= SYM_MARGIN and n_bad / ref_sym.size <= SYM_RATE
    del margin, diff, ref_sym
    again = oracle.pack(sym_gpu, C, bits, d, ln, oracle.canonical_codes(ln), cap=n + 4096)
    assert len(again) == n and (got == again).all()
    assert pbits == int(ln[sym_gpu].astype(np.uint64).sum())
    # same symbols as the encoder that builds its own table -> the same reconstruction, bit for bit
    stream_a, _ = fmtc.encode(basis, x_d, bits, synth.NHWC)
    xhat_a, err_a = fmtc.decode(basis, stream_a, x.shape, bits, synth.NHWC)
    torch.cuda.synchronize()
    assert int(err_a.item()) == 0 and torch.equal(xhat, xhat_a)
    # and so does the decoder that takes its tables from the handle
    xhat_s, err_s = fmtc.decode_static(basis, table, stream, x.shape, synth.NHWC)
    torch.cuda.synchronize()
    assert int(err_s.item()) == 0 and torch.equal(xhat_s, xhat)


# planar (NCHW) tensors at full size: one shape per kernel family (wavefront per tile, tiled matrix product)
PLANAR = [("resnet18_stage2_c128_28", 6), ("resnet18_stage3_c256_14", 4)]


@pytest.mark.parametrize("name,bits", PLANAR, ids=[f"{n}_b{b}" for n, b in PLANAR])
def test_full_size_planar_layout(fmtc, oracle, name, bits):
    wl = synth.WORKLOADS[name]
    C = wl["C"]
    calib, x = synth.workload(name, seed=0)
    T, mu, A = fit_on_host(oracle, calib, C)
    d = oracle.delta(A, bits)
    P = x.size // C
    xs = synth.to_layout(x, synth.NCHW)
    basis = fmtc.basis_import(T, mu, A)
    stream, nbytes = fmtc.encode(basis, torch.from_numpy(xs).cuda(), bits, synth.NCHW)
    xhat, err = fmtc.decode(basis, stream, xs.shape, bits, synth.NCHW)
    torch.cuda.synchronize()
    n = int(nbytes.item())
    got = stream[:n].cpu().numpy()
    assert int(err.item()) == 0
    sym_gpu, d2, _ = oracle.unpack(got, P, C, bits)
    assert d2 == d
    ref_sym, margin = oracle.quantize(oracle.project(xs, T, mu, synth.NCHW), d, bits, want_margin=True)
    diff = sym_gpu != ref_sym
    n_bad = int(diff.sum())
    if n_bad:
        assert margin[diff].max() <= SYM_MARGIN and n_bad / ref_sym.size <= SYM_RATE
    h = oracle.histogram(sym_gpu, bits)
    ln = oracle.huffman_lengths(h[: 1 << bits])
    again = oracle.pack(sym_gpu, C, bits, d, ln, oracle.canonical_codes(ln))
    assert len(again) == n and (got == again).all()
    ref = oracle.reconstruct(sym_gpu, xs.shape, T, mu, d, bits, synth.NCHW)
    assert float(np.abs(xhat.cpu().numpy().astype(np.float64) - ref).max()) <= RECON_TOL


def test_full_size_8bit_path(fmtc, oracle):
    """The 8-bit basis and activations at the stage-2 benchmark size: every output equals the oracle's."""
    name, bits = "resnet18_stage2_c128_28", 6
    C = synth.WORKLOADS[name]["C"]
    calib, x = synth.workload(name, seed=0)
    T, mu, A = fit_on_host(oracle, calib, C)
    d = oracle.delta(A, bits)
    sx = np.float32(float(x.max()) / 255.0)
    xq = np.clip(np.rint(x / sx), 0, 255).astype(np.uint8)
    Tq, sT, mf = oracle.basis8(T, mu, sx)
    b8 = fmtc.Basis8(fmtc.basis_import(T, mu, A), sx)
    stream, nbytes = fmtc.encode_u8(b8, torch.from_numpy(xq).cuda(), bits)
    out, err = fmtc.decode_u8(b8, stream, xq.shape, bits)
    torch.cuda.synchronize()
    assert int(err.item()) == 0
    sym = oracle.quantize_u8(xq, Tq, sT, mf, sx, d, bits)
    ln = oracle.huffman_lengths(oracle.histogram(sym, bits)[: 1 << bits])
    ref = oracle.pack(sym, C, bits, d, ln, oracle.canonical_codes(ln))
    n = int(nbytes.item())
    assert n == len(ref) and (stream[:n].cpu().numpy() == ref).all()
    assert (out.cpu().numpy() == oracle.reconstruct_u8(sym, xq.shape, Tq, sT, mf, sx, d, bits)).all()
