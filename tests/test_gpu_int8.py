"""GPU parity of the 8-bit path (section 3.1 'Linear transform': PCA matrix at 8 bits; section 5: 8-bit
activations) through the C ABI against the oracle's integer arithmetic: everything is bit-exact."""
import numpy as np
import pytest

from paper_1905_10830_amd import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fmtc():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1905_10830_amd import binding

    binding.load_library()
    return binding


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def make_case(oracle, C, H, W, n, rank, act, seed):
    """uint8 activations (NHWC), their scale, and an fp32 basis fitted on the dequantized calibration images."""
    s = synth.FeatureMapStream(C, H, W, rank, act, seed)
    x = s.images(n)
    lo = min(0.0, float(x.min()))
    sx = np.float32((float(x.max()) - lo) / 255.0)
    xq = np.clip(np.rint((x - lo) / sx), 0, 255).astype(np.uint8)
    deq = xq.astype(np.float32) * sx
    if C <= 64:
        T, mu, eig, A = oracle.fit(deq)
    else:
        mean, cov = oracle.covariance(deq)
        w, v = np.linalg.eigh(cov)
        T = np.ascontiguousarray(v[:, ::-1].T).astype(np.float32)
        mu = mean.astype(np.float32)
        A = oracle.dynamic_range(deq, T[0], mu)
    return xq, sx, T, mu, A


# (C, H, W, images, rank, act, bits): register-resident and reloading kernels, vector and byte paths, ragged tiles
CASES = [
    (128, 28, 28, 2, 32, "relu", 6),
    (64, 19, 17, 2, 16, "relu", 8),
    (128, 7, 9, 3, 32, "relu6", 4),
    (24, 9, 9, 2, 6, "relu", 5),      # C % 16 != 0, C % 8 == 0
    (50, 10, 10, 2, 10, "relu", 5),   # byte paths
    (3, 17, 5, 1, 2, "none", 2),
    (144, 6, 7, 2, 18, "relu6", 5),   # more than 8 contraction steps: the reloading kernel
    (256, 7, 7, 3, 64, "relu", 4),
    (200, 5, 5, 2, 25, "relu", 3),
]
IDS = [f"C{c[0]}_{c[1]}x{c[2]}_n{c[3]}_b{c[6]}" for c in CASES]


@pytest.mark.parametrize("layout", [synth.NHWC, synth.NCHW], ids=["nhwc", "nchw"])
@pytest.mark.parametrize("case", CASES, ids=IDS)
def test_u8_path_is_bit_exact(fmtc, oracle, case, layout):
    C, H, W, n, rank, act, bits = case
    xq, sx, T, mu, A = make_case(oracle, C, H, W, n, rank, act, 700 + C)
    xs = synth.to_layout(xq, layout)
    d = oracle.delta(A, bits)
    Tq, sT, mf = oracle.basis8(T, mu, sx)
    b8 = fmtc.Basis8(fmtc.basis_import(T, mu, A), sx)
    Tq_g, sT_g, mf_g, sx_g, A_g = b8.export()
    assert np.array_equal(Tq_g, Tq) and sT_g == sT and np.array_equal(mf_g, mf) and sx_g == sx and A_g == A
    want = oracle.quantize_u8(xs, Tq, sT, mf, sx, d, bits, layout)
    sym = fmtc.quantize_u8(b8, dev(xs), bits, layout)
    torch.cuda.synchronize()
    got = sym.cpu().numpy()
    assert np.array_equal(got, want), f"{int((got != want).sum())} symbols differ"
    # inverse, on the oracle's symbols and on arbitrary ones
    rng = np.random.default_rng(C)
    for s_in in (want, rng.integers(0, 1 << bits, size=want.shape).astype(np.uint8)):
        ref = oracle.reconstruct_u8(s_in, xs.shape, Tq, sT, mf, sx, d, bits, layout)
        out = fmtc.reconstruct_u8(b8, dev(s_in), xs.shape, bits, layout)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), ref)
    # whole encoder and decoder: the stream is the oracle's packing of those symbols with their own table
    h = oracle.histogram(want, bits)
    ln = oracle.huffman_lengths(h[: 1 << bits])
    ref_stream = oracle.pack(want, C, bits, d, ln, oracle.canonical_codes(ln))
    stream, nbytes = fmtc.encode_u8(b8, dev(xs), bits, layout)
    torch.cuda.synchronize()
    nb = int(nbytes.item())
    assert nb == len(ref_stream) and np.array_equal(stream[:nb].cpu().numpy(), ref_stream)
    out, err = fmtc.decode_u8(b8, stream, xs.shape, bits, layout)
    torch.cuda.synchronize()
    assert int(err.item()) == 0
    assert np.array_equal(out.cpu().numpy(), oracle.reconstruct_u8(want, xs.shape, Tq, sT, mf, sx, d, bits, layout))


def test_u8_codec_quality_and_errors(fmtc, oracle):
    """The 8-bit path is a usable codec (error of the order of the quantizer's plus the grids'), and the entry
    points refuse what does not fit."""
    xq, sx, T, mu, A = make_case(oracle, 64, 14, 14, 4, 16, "relu", 41)
    basis = fmtc.basis_import(T, mu, A)
    b8 = fmtc.Basis8(basis, sx)
    x_d = dev(xq)
    stream, nbytes = fmtc.encode_u8(b8, x_d, 6)
    out, err = fmtc.decode_u8(b8, stream, xq.shape, 6)
    torch.cuda.synchronize()
    assert int(err.item()) == 0
    step = float(fmtc.delta(A, 6))
    mse = float((((out.cpu().numpy().astype(np.float64) - xq) * float(sx)) ** 2).mean())
    assert mse < 2.0 * step * step / 12 + float(sx) ** 2 / 6
    # fp32 path on the same data for comparison: the 8-bit basis costs little
    s32, n32 = fmtc.encode(basis, dev(xq.astype(np.float32) * sx), 6)
    torch.cuda.synchronize()
    assert abs(int(nbytes.item()) - int(n32.item())) < 0.05 * int(n32.item())
    with pytest.raises(fmtc.FmtcError) as e:
        fmtc.Basis8(basis, 0.0)
    assert e.value.status == fmtc.EINVAL
    with pytest.raises(fmtc.FmtcError) as e:
        fmtc.quantize_u8(b8, dev(np.zeros((1, 4, 4, 32), np.uint8)), 6)
    assert e.value.status == fmtc.EINVAL
    with pytest.raises(fmtc.FmtcError) as e:
        fmtc.quantize_u8(b8, x_d, 9)
    assert e.value.status == fmtc.EINVAL
    # up to 128 channels the decoder needs no workspace; wider tensors refuse one that cannot hold the symbols
    xw, sxw, Tw, muw, Aw = make_case(oracle, 144, 6, 7, 2, 18, "relu6", 43)
    b8w = fmtc.Basis8(fmtc.basis_import(Tw, muw, Aw), sxw)
    sw, nw = fmtc.encode_u8(b8w, dev(xw), 5)
    with pytest.raises(fmtc.FmtcError) as e:
        fmtc.decode_u8(b8w, sw, xw.shape, 5, workspace=torch.empty(1024, dtype=torch.uint8, device="cuda"))
    assert e.value.status == fmtc.EBUFSIZE
    # a damaged stream is flagged and nothing faults
    bad = stream.clone()
    bad[2] ^= 0x55
    out2, err2 = fmtc.decode_u8(b8, bad, xq.shape, 6)
    torch.cuda.synchronize()
    assert int(err2.item()) != 0


@pytest.mark.parametrize("name,bits", [("resnet18_stage2_c128_28", 6), ("cfg0_c64_56", 8),
                                       ("resnet18_n256_c64_56", 6)])  # (the last: four wavefronts per SIMD)
def test_u8_path_at_full_size(fmtc, oracle, name, bits):
    """The benchmark's tensors as 8-bit activations, in the launch configuration the benchmark times: symbols,
    stream and decoded activations equal the oracle's everywhere."""
    calib, data = synth.workload(name, seed=0)
    C = data.shape[-1]
    sx = np.float32(float(data.max()) / 255.0)
    xq = np.clip(np.rint(data / sx), 0, 255).astype(np.uint8)
    basis = fmtc.fit_basis(dev(calib))
    T, mu, eig, A = basis.export()
    d = oracle.delta(A, bits)
    Tq, sT, mf = oracle.basis8(T, mu, sx)
    b8 = fmtc.Basis8(basis, sx)
    want = oracle.quantize_u8(xq, Tq, sT, mf, sx, d, bits)
    x_d = dev(xq)
    sym = fmtc.quantize_u8(b8, x_d, bits)
    stream, nbytes = fmtc.encode_u8(b8, x_d, bits)
    out, err = fmtc.decode_u8(b8, stream, xq.shape, bits)
    torch.cuda.synchronize()
    assert int(err.item()) == 0
    assert np.array_equal(sym.cpu().numpy(), want)
    h = oracle.histogram(want, bits)
    ln = oracle.huffman_lengths(h[: 1 << bits])
    ref_stream = oracle.pack(want, C, bits, d, ln, oracle.canonical_codes(ln))
    nb = int(nbytes.item())
    assert nb == len(ref_stream) and np.array_equal(stream[:nb].cpu().numpy(), ref_stream)
    assert np.array_equal(out.cpu().numpy(), oracle.reconstruct_u8(want, xq.shape, Tq, sT, mf, sx, d, bits))
