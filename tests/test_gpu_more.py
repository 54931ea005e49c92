"""More GPU parity: the bit depths of the inference-shaped sweep, chunk sizes other than the nominal one through
the whole encoder and decoder, a planar (NCHW) tensor at a full benchmark size, and damaged streams through the
fused decoder (flags, never faults)."""
import numpy as np
import pytest

from paper_1905_10830_amd import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

SYM_MARGIN = 1e-4
SYM_RATE = 1e-6
RECON_TOL = 1e-4


@pytest.fixture(scope="module")
def fmtc():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1905_10830_amd import binding

    binding.load_library()
    return binding


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def roundtrip(fmtc, oracle, x, T, mu, A, bits, layout, chunk_syms=4096):
    """Encode + decode on the GPU, every output against the oracle.  x: storage array in `layout`."""
    C = T.shape[0]
    P = x.size // C
    d = oracle.delta(A, bits)
    basis = fmtc.basis_import(T, mu, A)
    stream, nbytes = fmtc.encode(basis, dev(x), bits, layout, chunk_syms=chunk_syms)
    xhat, err = fmtc.decode(basis, stream, x.shape, bits, layout)
    torch.cuda.synchronize()
    n = int(nbytes.item())
    got = stream[:n].cpu().numpy()
    assert int(err.item()) == 0
    sym_gpu, d2, pbits = oracle.unpack(got, P, C, bits)
    assert d2 == d
    ref_sym, margin = oracle.quantize(oracle.project(x, T, mu, layout), d, bits, want_margin=True)
    diff = sym_gpu != ref_sym
    if diff.any():
        assert margin[diff].max() <= SYM_MARGIN and diff.mean() <= SYM_RATE
    h = oracle.histogram(sym_gpu, bits)
    ln = oracle.huffman_lengths(h[: 1 << bits])
    again = oracle.pack(sym_gpu, C, bits, d, ln, oracle.canonical_codes(ln), chunk_syms=chunk_syms)
    assert len(again) == n and (got == again).all()
    ref = oracle.reconstruct(sym_gpu, x.shape, T, mu, d, bits, layout)
    assert np.abs(xhat.cpu().numpy().astype(np.float64) - ref).max() <= RECON_TOL
    return got


@pytest.mark.parametrize("bits", [8, 6, 4, 3, 2])
@pytest.mark.parametrize("C,hw,rank", [(64, 28, 16), (128, 14, 32)], ids=["C64", "C128"])
def test_bit_depth_sweep(fmtc, oracle, C, hw, rank, bits):
    s = synth.FeatureMapStream(C, hw, hw, rank, "relu", seed=500 + C)
    calib, x = s.images(2), s.images(5)
    T, mu, _, A = oracle.fit(calib)
    roundtrip(fmtc, oracle, x, T, mu, A, bits, synth.NHWC)


@pytest.mark.parametrize("chunk_syms", [64, 1000, 2048, 4000])
@pytest.mark.parametrize("C", [32, 128, 256])
def test_other_chunk_sizes(fmtc, oracle, C, chunk_syms):
    """The decoder sizes its first requests for the nominal chunk size; any other chunk size must still decode."""
    s = synth.FeatureMapStream(C, 9, 11, max(2, C // 4), "relu", seed=600 + C)
    calib, x = s.images(1), s.images(3)
    if C <= 160:
        T, mu, _, A = oracle.fit(calib)
    else:
        mean, cov = oracle.covariance(calib)
        w, v = np.linalg.eigh(cov)
        T = np.ascontiguousarray(v[:, ::-1].T).astype(np.float32)
        mu = mean.astype(np.float32)
        A = np.float32(np.abs(oracle.project(calib, T, mu)[:, 0]).max())
    roundtrip(fmtc, oracle, x, T, mu, A, 5, synth.NHWC, chunk_syms=chunk_syms)


def test_planar_layout_at_full_size(fmtc, oracle):
    """The ResNet-18 stage-2 batch stored NCHW."""
    calib, data = synth.workload("resnet18_stage2_c128_28", seed=0)
    T, mu, _, A = oracle.fit(calib)
    roundtrip(fmtc, oracle, synth.to_layout(data, synth.NCHW), T, mu, A, 6, synth.NCHW)


def test_damaged_streams_through_the_fused_decoder(fmtc, oracle):
    s = synth.FeatureMapStream(64, 12, 12, 16, "relu", seed=7)
    calib, x = s.images(1), s.images(4)
    T, mu, _, A = oracle.fit(calib)
    good = roundtrip(fmtc, oracle, x, T, mu, A, 5, synth.NHWC)
    basis = fmtc.basis_import(T, mu, A)

    def flag(stream, nbytes=None):
        xhat, err = fmtc.decode(basis, dev(stream), x.shape, 5, synth.NHWC, nbytes=nbytes)
        torch.cuda.synchronize()
        return int(err.item())

    assert flag(good) == 0
    bad = good.copy(); bad[0] ^= 0xFF
    assert flag(bad) & fmtc.ERR_HEADER
    assert flag(good, nbytes=len(good) - 8) & fmtc.ERR_HEADER
    assert flag(good, nbytes=200) & fmtc.ERR_HEADER
    bad = good.copy(); bad[64:320] = 1  # 256 one-bit codes: not a prefix code
    assert flag(bad) & fmtc.ERR_TABLE
    bad = good.copy(); bad[320 + 4: 320 + 8] = 0xFF  # second chunk offset far past the payload
    assert flag(bad) & fmtc.ERR_OFFSETS
    # random damage to the payload must never fault (it may or may not be detectable)
    rng = np.random.default_rng(3)
    info = fmtc.stream_info(good[:64])
    pay0 = len(good) - 4 * ((info["payload_bits"] + 31) // 32)
    for _ in range(8):
        bad = good.copy()
        idx = rng.integers(max(pay0, 320), len(good), size=16)
        bad[idx] = rng.integers(0, 256, size=16, dtype=np.uint8)
        flag(bad)


@pytest.mark.parametrize("layout", [synth.NHWC, synth.NCHW], ids=["nhwc", "nchw"])
@pytest.mark.parametrize("C", [320, 960])
def test_wide_decoder_walking_its_channel_groups(fmtc, oracle, C, layout, monkeypatch):
    """More than 256 channels: a tile's channel groups normally go to workgroups of their own; with more tiles than
    the device holds at once one workgroup walks them in turn.  That second way is forced here on a small tensor
    and must give the same tensor, to the bit, as the first."""
    s = synth.FeatureMapStream(C, 9, 11, max(8, C // 8), "relu", 1200 + C)
    x = synth.to_layout(s.images(3), layout)
    mean, cov = oracle.covariance(x, layout)
    w, v = np.linalg.eigh(cov)
    T = np.ascontiguousarray(v[:, ::-1].T).astype(np.float32)
    mu = mean.astype(np.float32)
    A = np.float32(np.abs(oracle.project(x, T, mu, layout)[:, 0]).max())
    basis = fmtc.basis_import(T, mu, A)
    x_d = torch.from_numpy(x).cuda()
    stream, nbytes = fmtc.encode(basis, x_d, 5, layout)
    a, ea = fmtc.decode(basis, stream, x.shape, 5, layout)
    torch.cuda.synchronize()
    fmtc.test_option(fmtc.TEST_DECODE_ONE_ROW, 1)
    try:
        b, eb = fmtc.decode(basis, stream, x.shape, 5, layout)
        torch.cuda.synchronize()
    finally:
        fmtc.test_option(fmtc.TEST_DECODE_ONE_ROW, 0)
    assert int(ea.item()) == 0 and int(eb.item()) == 0 and torch.equal(a, b)
    sym, d, _ = oracle.unpack(stream[: int(nbytes.item())].cpu().numpy(), x.size // C, C, 5)
    ref = oracle.reconstruct(sym, x.shape, T, mu, d, 5, layout)
    assert np.abs(b.cpu().numpy().astype(np.float64) - ref).max() <= 1e-4


@pytest.mark.parametrize("layout", [synth.NHWC, synth.NCHW], ids=["nhwc", "nchw"])
def test_wide_projection_with_more_tiles_than_compute_units(fmtc, oracle, layout):
    """256 channels, 18000 pixels: 141 x 2 workgroup tiles, which takes the 4-wavefront form of the tiled
    projection (small tensors take the 8-wavefront form), including a ragged last pixel tile."""
    C, bits = 256, 4
    s = synth.FeatureMapStream(C, 30, 30, 64, "relu", 1400)
    calib, data = s.images(2), s.images(20)
    x = synth.to_layout(data, layout)
    mean, cov = oracle.covariance(synth.to_layout(calib, layout), layout)
    w, v = np.linalg.eigh(cov)
    T = np.ascontiguousarray(v[:, ::-1].T).astype(np.float32)
    mu = mean.astype(np.float32)
    A = np.float32(np.abs(oracle.project(synth.to_layout(calib, layout), T, mu, layout)[:, 0]).max())
    d = oracle.delta(A, bits)
    ref_sym, margin = oracle.quantize(oracle.project(x, T, mu, layout), d, bits, want_margin=True)
    basis = fmtc.basis_import(T, mu, A)
    sym, hist = fmtc.quantize(basis, torch.from_numpy(x).cuda(), bits, layout)
    torch.cuda.synchronize()
    sym, hist = sym.cpu().numpy().reshape(ref_sym.shape), hist.cpu().numpy()
    diff = sym != ref_sym
    n_bad = int(diff.sum())
    if n_bad:
        assert margin[diff].max() <= 1e-4 and n_bad / ref_sym.size <= 1e-6
    assert hist.tolist() == np.bincount(sym.reshape(-1), minlength=256).tolist()


def test_rate_distortion_sweep_against_the_oracle(fmtc, oracle):
    """The sweep utility's numbers are the oracle's: entropy and rate from identical histograms, distortion from
    the fp64 reconstruction of the same symbols; and they behave as section 3.1 says (H <= R < H + 1), with the
    distortion near Delta^2 / 12 per coefficient while the quantizer does not clamp."""
    from paper_1905_10830_amd import rd

    s = synth.FeatureMapStream(64, 12, 12, 16, "relu", 1500)
    calib, x = s.images(2), s.images(3)
    T, mu, eig, A = oracle.fit(calib)
    basis = fmtc.basis_import(T, mu, A)
    rows = rd.sweep(basis, torch.from_numpy(x).cuda(), bits_list=(8, 6, 4, 2))
    prev_rate, prev_mse = None, None
    for r in rows:
        bits = r["bits"]
        d = oracle.delta(A, bits)
        assert r["delta"] == float(d)
        enc = oracle.encode(x, T, mu, d, bits, want_margin=True)
        h = enc["hist"][: 1 << bits]
        ln = oracle.huffman_lengths(h)
        # a symbol or two may sit on a rounding boundary: allow the histogram to move by that much
        assert abs(r["entropy"] - oracle.entropy(h)) < 1e-3
        assert abs(r["rate"] - float((h * ln.astype(np.uint64)).sum()) / x.size) < 1e-3
        assert r["entropy"] <= r["rate"] + 1e-9 < r["entropy"] + 1.0
        ref_hat, _ = oracle.decode(enc["stream"], x.shape, T, mu, bits)
        assert abs(r["mse"] - oracle.mse(x, ref_hat)) <= 1e-3 * oracle.mse(x, ref_hat) + 1e-9
        if prev_rate is not None:
            assert r["rate"] < prev_rate and r["mse"] > prev_mse  # fewer bits: lower rate, higher distortion
        prev_rate, prev_mse = r["rate"], r["mse"]
    assert rows[0]["mse"] < 1.3 * rows[0]["delta"] ** 2 / 12


def test_encoders_on_two_streams_share_the_device(fmtc):
    """Two encoder calls of a tensor with more chunk groups than the pack kernel has workgroups, in flight on
    two HIP streams at once: neither kernel has the device to itself, so not all of its workgroups are resident
    together.  Every call must still give the one-stream result (groups are claimed from a counter there, so a
    wait never depends on a workgroup that has not started)."""
    torch.manual_seed(5)
    C, bits = 128, 6
    calib = torch.randn(8, 28, 28, C, device="cuda").relu()
    x = (torch.randn(256, 28, 28, C, device="cuda") * torch.linspace(2.0, 0.05, C, device="cuda")).relu()
    basis = fmtc.fit_basis(calib)
    P = 256 * 28 * 28
    assert (P * C // 4096 + 3) // 4 > 1024          # more groups than workgroups
    ref, ref_n = fmtc.encode(basis, x, bits)
    torch.cuda.synchronize()
    n = int(ref_n.item())
    assert fmtc.stream_info(ref[:64].cpu().numpy())["stream_bytes"] == n
    side = [torch.cuda.Stream(), torch.cuda.Stream()]
    outs = []
    for rep in range(3):
        for st in side:
            with torch.cuda.stream(st):
                outs.append(fmtc.encode(basis, x, bits))
    torch.cuda.synchronize()
    for stream, nbytes in outs:
        assert int(nbytes.item()) == n
        assert torch.equal(stream[:n], ref[:n])
    xhat, err = fmtc.decode(basis, outs[-1][0], x.shape, bits)
    torch.cuda.synchronize()
    assert int(err.item()) == 0


def test_small_tensor_encoders_on_two_streams(fmtc):
    """The same for a tensor that takes the one-kernel packer (at most 1024 chunk groups, workgroup g packs group g
    and waits for the groups before it through the look-back words): calls in flight on two HIP streams give the
    one-stream bytes.  What the packer relies on there: the workgroups of a launch start in index order, so the
    group a workgroup waits for belongs to a workgroup that was dispatched before it; if that ever failed to hold,
    a wait would run into its limit and the stream would come out marked invalid, which this test would see."""
    torch.manual_seed(6)
    C, bits = 128, 6
    calib = torch.randn(8, 28, 28, C, device="cuda").relu()
    x = (torch.randn(64, 28, 28, C, device="cuda") * torch.linspace(2.0, 0.05, C, device="cuda")).relu()
    basis = fmtc.fit_basis(calib)
    P = 64 * 28 * 28
    assert (P * C // 4096 + 3) // 4 <= 1024
    ref, ref_n = fmtc.encode(basis, x, bits)
    torch.cuda.synchronize()
    n = int(ref_n.item())
    assert fmtc.stream_info(ref[:64].cpu().numpy())["stream_bytes"] == n
    side = [torch.cuda.Stream(), torch.cuda.Stream()]
    outs = []
    for rep in range(4):
        for st in side:
            with torch.cuda.stream(st):
                outs.append(fmtc.encode(basis, x, bits))
    torch.cuda.synchronize()
    for stream, nbytes in outs:
        assert int(nbytes.item()) == n
        assert torch.equal(stream[:n], ref[:n])


@pytest.mark.parametrize("layout", [synth.NHWC, synth.NCHW], ids=["nhwc", "nchw"])
@pytest.mark.parametrize("C,rank", [(64, 16), (128, 32), (144, 18), (160, 20), (256, 64)], ids=["C64", "C128", "C144", "C160", "C256"])
def test_pixels_too_large_for_f16(fmtc, oracle, C, rank, layout):
    """Activations far outside the range the split-f16 products cover (a component beyond the largest f16 number
    turns into infinity on the way into the matrix cores): such a pixel's coefficients are all decided in fp64, so
    the symbols still equal the oracle's, the pixels around it are untouched, and the histogram, the container and
    the decoded tensor stay consistent.  One pixel just below the limit of the exact treatment as well."""
    s = synth.FeatureMapStream(C, 9, 11, rank, "relu", seed=900 + C)
    calib, x = s.images(1), s.images(3)
    if C <= 160:
        T, mu, _, A = oracle.fit(calib)
    else:
        mean, cov = oracle.covariance(calib)
        w, v = np.linalg.eigh(cov)
        T = np.ascontiguousarray(v[:, ::-1].T).astype(np.float32)
        mu = mean.astype(np.float32)
        A = np.float32(np.abs(oracle.project(calib, T, mu)[:, 0]).max())
    x = x.copy()
    flat = x.reshape(-1, C)
    flat[5, 3] = 1.0e5          # beyond f16
    flat[5, C - 1] = -2.5e5
    flat[40, 0] = 3.0e7         # far beyond: its products overflow fp32 accumulation of the others' scale
    flat[77, C // 2] = 7.0e4
    flat[130, 1] = 2.0e4        # large, still inside f16: the ordinary path with a wide exact-decision band
    flat[131] = 900.0           # |x - mu|_2 close to the limit of the exact treatment (about 3e4) at 1e3 per channel
    xs = synth.to_layout(x, layout)
    roundtrip(fmtc, oracle, xs, T, mu, A, 6, layout)


@pytest.mark.parametrize("C,hw,N", [(64, 56, 64), (128, 28, 128), (144, 56, 24)], ids=["C64", "C128", "C144"])
def test_damaged_streams_through_the_many_wavefront_decoders(fmtc, C, hw, N):
    """Tensors of more than 3000 chunks take the chunk decoder's variants with three and four wavefronts per SIMD
    (payload straight into LDS, three table entries per stream read, part of the basis read from global memory).
    Damage to the payload, the run sizes and the chunk offsets of such a stream must end in a flag or in garbage,
    never in an access outside the buffers; the undamaged stream decodes without a flag before and after."""
    torch.manual_seed(11)
    calib = torch.randn(4, hw, hw, C, device="cuda").relu()
    x = (torch.randn(N, hw, hw, C, device="cuda") * torch.linspace(2.0, 0.05, C, device="cuda")).relu()
    P = N * hw * hw
    assert (P + 4096 // C - 1) // (4096 // C) > (3072 if C <= 64 else 2048)
    basis = fmtc.fit_basis(calib)
    stream, nbytes = fmtc.encode(basis, x, 6)
    ref, err = fmtc.decode(basis, stream, x.shape, 6)
    torch.cuda.synchronize()
    assert int(err.item()) == 0
    n = int(nbytes.item())
    good = stream[:n].cpu().numpy()
    info = fmtc.stream_info(good[:64])
    n_chunks = info["n_chunks"]
    off_co = 64 + 256
    off_sub = (off_co + 4 * (n_chunks + 1) + 15) // 16 * 16
    spc = (4096 // C * C + 63) // 64
    off_pay = (off_sub + 2 * n_chunks * spc + 15) // 16 * 16
    rng = np.random.default_rng(C)

    def run(bad):
        out, e = fmtc.decode(basis, dev(bad), x.shape, 6)
        torch.cuda.synchronize()
        return int(e.item())

    # payload bytes at random places
    bad = good.copy()
    idx = rng.integers(off_pay, n, size=4000)
    bad[idx] = rng.integers(0, 256, size=4000, dtype=np.uint8)
    run(bad)
    # run sizes: some far too large, some zero
    bad = good.copy()
    sub = bad[off_sub:off_sub + 2 * n_chunks * spc].view(np.uint16)
    pick = rng.integers(0, sub.size, size=2000)
    sub[pick[:1000]] = 0xFFFF
    sub[pick[1000:]] = 0
    run(bad)
    # chunk offsets: two neighbours swapped (decreasing), one beyond the payload
    bad = good.copy()
    co = bad[off_co:off_co + 4 * (n_chunks + 1)].view(np.uint32)
    co[[100, 101]] = co[[101, 100]]
    co[n_chunks // 2] = 0xFFFFFFF0
    assert run(bad) & fmtc.ERR_OFFSETS
    # the payload cut short of what the header announces
    out, e = fmtc.decode(basis, dev(good), x.shape, 6, nbytes=n - 4096)
    torch.cuda.synchronize()
    assert int(e.item()) & fmtc.ERR_HEADER
    # and the good stream still decodes to the same tensor
    again, err = fmtc.decode(basis, dev(good), x.shape, 6)
    torch.cuda.synchronize()
    assert int(err.item()) == 0 and torch.equal(again, ref)
