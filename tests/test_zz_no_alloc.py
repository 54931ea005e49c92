"""fmtc_encode_noalloc (the encoder with its workspace in the library's own device array, for callers that cannot
allocate) against fmtc_encode with a caller workspace: the two run the same kernels, so the containers must be equal
byte for byte.  Two calls in a row on the same GPU, the second with a smaller tensor (the array keeps the first
call's contents), then the first again; the oracle's container for the same symbols closes the chain."""
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


def _case(oracle, C, H, W, n, rank, seed):
    s = synth.FeatureMapStream(C, H, W, rank, "relu", seed)
    calib, data = s.images(2), s.images(n)
    T, mu, _, A = oracle.fit(calib)
    return data, T, mu, A


def _both(fmtc, basis, x_d, bits, poison):
    n, h, w, c = x_d.shape
    cap = fmtc.encode_bound(n * h * w, c, bits)
    ref, ref_n = fmtc.encode(basis, x_d, bits)
    out = torch.full((cap,), poison, dtype=torch.uint8, device="cuda")
    out_n = torch.zeros(1, dtype=torch.int64, device="cuda")
    fmtc.encode_noalloc(basis, x_d, bits, out, out_n)
    torch.cuda.synchronize()
    k = int(ref_n.item())
    assert int(out_n.item()) == k
    a, b = ref[:k].cpu().numpy(), out[:k].cpu().numpy()
    assert (a == b).all(), f"first differing byte {int(np.argmax(a != b))}"
    assert (out[k:] == poison).all(), "bytes past the stream were written"
    return b


def test_noalloc_encoder_equals_the_workspace_encoder(fmtc, oracle):
    big, Tb, mub, Ab = _case(oracle, 128, 28, 28, 5, 32, 7)     # 501 760 values, several chunk groups
    small, Ts, mus, As = _case(oracle, 64, 9, 7, 2, 16, 8)      # 8 064 values: ragged last chunk
    bb, bs = fmtc.basis_import(Tb, mub, Ab), fmtc.basis_import(Ts, mus, As)
    xb, xs = torch.from_numpy(big).cuda(), torch.from_numpy(small).cuda()
    first = _both(fmtc, bb, xb, 6, 0xA5)
    second = _both(fmtc, bs, xs, 4, 0x5A)   # smaller input right after: nothing of the first call may leak in
    again = _both(fmtc, bb, xb, 6, 0xC3)
    assert (first == again).all()
    # the container is the oracle's packing of the symbols it carries
    for got, x, C, bits, A in ((first, big, 128, 6, Ab), (second, small, 64, 4, As)):
        sym, _, _ = oracle.unpack(got, x.size // C, C, bits)
        ln = oracle.huffman_lengths(oracle.histogram(sym, bits)[: 1 << bits])
        ref = oracle.pack(sym, C, bits, oracle.delta(A, bits), ln, oracle.canonical_codes(ln))
        assert len(ref) == len(got) and (ref == got).all()


def test_noalloc_encoder_rejects_what_does_not_fit(fmtc, oracle):
    data, T, mu, A = _case(oracle, 64, 8, 8, 1, 16, 9)
    basis = fmtc.basis_import(T, mu, A)
    # 8 M values need more scratch than the library's array holds: refused on the host, nothing is launched
    N, C, H, W = 512, 64, 16, 16
    assert fmtc.workspace_size(N * H * W, C, 6) > fmtc.NOALLOC_SCRATCH_BYTES
    x = torch.zeros((N, H, W, C), dtype=torch.float32, device="cuda")
    out = torch.zeros(fmtc.encode_bound(N * H * W, C, 6), dtype=torch.uint8, device="cuda")
    out_n = torch.zeros(1, dtype=torch.int64, device="cuda")
    with pytest.raises(fmtc.FmtcError) as e:
        fmtc.encode_noalloc(basis, x, 6, out, out_n)
    assert e.value.status == fmtc.EBUFSIZE and "too large" in str(e.value)
    torch.cuda.synchronize()
    assert int(out.max().item()) == 0
