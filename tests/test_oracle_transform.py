"""Pins for the oracle's fit, projection, quantizer and reconstruction
(section 3 'Transform-Domain Compression'; section 3.1 'Linear transform', 'Quantization')."""
import numpy as np
import pytest

from paper_1905_10830_amd import synth


def _nhwc(points):
    """[P, C] rows -> a [1, P, 1, C] channels-last tensor."""
    a = np.asarray(points, np.float32)
    return a.reshape(1, a.shape[0], 1, a.shape[1])


def test_fit_2x2_closed_form(oracle):
    """Sigma = [[2,1],[1,2]] has eigenvalues 3 and 1 with eigenvectors (1,1)/sqrt2 and (1,-1)/sqrt2."""
    r3 = np.sqrt(3.0)
    pts = [(r3, r3), (-r3, -r3), (1, -1), (-1, 1)]
    mean, cov = oracle.covariance(_nhwc(pts))
    assert np.allclose(mean, 0, atol=1e-7)
    assert np.allclose(cov, [[2, 1], [1, 2]], atol=1e-6)
    T, mu, eig, A = oracle.fit(_nhwc(pts))
    assert np.allclose(eig, [3, 1], atol=1e-6)
    s = 1 / np.sqrt(2)
    assert np.allclose(T, [[s, s], [s, -s]], atol=1e-6)
    # range: max |y0| = |(sqrt3+sqrt3)/sqrt2| = sqrt6
    assert A == pytest.approx(np.sqrt(6.0), rel=1e-6)


def test_fit_diagonal_covariance_is_a_permutation(oracle):
    rng = np.random.default_rng(0)
    std = np.array([0.5, 3.0, 1.0, 2.0])
    # exactly uncorrelated, exactly centred: +-std on one axis at a time
    pts = []
    for c, s in enumerate(std):
        for sign in (1, -1):
            v = np.zeros(4)
            v[c] = sign * s
            pts.append(v)
    T, mu, eig, A = oracle.fit(_nhwc(pts))
    assert np.allclose(mu, 0)
    assert np.allclose(eig, np.sort(std ** 2 * 2 / 8)[::-1])
    assert np.allclose(np.abs(T), np.eye(4)[[1, 3, 2, 0]])
    assert (T.sum(axis=1) > 0).all()  # sign rule: dominant entry positive


@pytest.mark.parametrize("layout", [synth.NHWC, synth.NCHW])
def test_fit_invariants_and_eigh_cross_check(oracle, layout):
    s = synth.FeatureMapStream(C=24, H=12, W=12, rank=6, act="none", seed=5)
    x = synth.to_layout(s.images(3), layout)
    mean, cov = oracle.covariance(x, layout)
    flat = (x if layout == synth.NHWC else np.transpose(x, (0, 2, 3, 1))).reshape(-1, 24).astype(np.float64)
    assert np.allclose(mean, flat.mean(0), atol=1e-12)
    assert np.allclose(cov, np.cov(flat.T, bias=True), atol=1e-12)
    T, eig = oracle.pca(cov)
    assert np.abs(T @ T.T - np.eye(24)).max() < 1e-12          # orthonormal, T^-1 = T^T
    D = T @ cov @ T.T
    assert np.abs(D - np.diag(np.diag(D))).max() < 1e-10 * eig[0]  # diagonalises Sigma
    assert (np.diff(eig) <= 1e-15).all()                        # descending
    assert eig.sum() == pytest.approx(np.trace(cov), rel=1e-12)
    w, v = np.linalg.eigh(cov)                                  # library routine, test side only
    assert np.allclose(eig, w[::-1], rtol=1e-10, atol=1e-14)
    for k in range(6):                                          # well separated leading components
        assert abs(abs(T[k] @ v[:, ::-1][:, k]) - 1) < 1e-9
    arg = np.abs(T).argmax(axis=1)
    assert (T[np.arange(24), arg] > 0).all()
    # rank 6 + 0.1 * noise, no activation: the 24-6 trailing eigenvalues sit at the noise floor 0.1^2
    assert 0.005 < eig[6:].min() and eig[6:].max() < 0.02 and eig[5] > 5 * eig[6]
    T32, mu32, eig2, A = oracle.fit(x, layout)
    assert np.abs(T32 - T).max() < 1e-7 and np.allclose(eig2, eig)
    y = oracle.project(x, T32, mu32, layout)
    assert A == np.float32(np.abs(y[:, 0]).max())


def test_projection_reconstructs_exactly_when_unquantized(oracle):
    """x = T^T (T (x - mu)) + mu for an orthonormal T (fp64 basis so only rounding remains)."""
    rng = np.random.default_rng(7)
    x = rng.standard_normal((2, 5, 4, 16)).astype(np.float32)
    q, _ = np.linalg.qr(rng.standard_normal((16, 16)))
    T = q.astype(np.float32)
    mu = rng.standard_normal(16).astype(np.float32)
    y = oracle.project(x, T, mu)
    direct = (x.reshape(-1, 16).astype(np.float64) - mu.astype(np.float64)) @ T.astype(np.float64).T
    assert np.abs(y - direct).max() < 1e-13
    back = y @ T.astype(np.float64) + mu.astype(np.float64)
    # T is orthonormal only to fp32 rounding after the cast
    assert np.abs(back - x.reshape(-1, 16)).max() < 5e-6
    Td = q  # the fp64 orthonormal matrix itself: exact to 1e-12
    y64 = (x.reshape(-1, 16).astype(np.float64) - mu) @ Td.T
    assert np.abs(y64 @ Td + mu - x.reshape(-1, 16)).max() < 1e-12


def test_project_is_not_transposed(oracle):
    """A non-symmetric T distinguishes T(x-mu) from T^T(x-mu)."""
    T = np.array([[0, 1, 0], [0, 0, 1], [1, 0, 0]], np.float32)  # y0 = x1, y1 = x2, y2 = x0
    mu = np.array([10, 20, 30], np.float32)
    x = _nhwc([[11, 22, 33]])
    assert oracle.project(x, T, mu).tolist() == [[2.0, 3.0, 1.0]]
    sym = np.array([[2 + 4, 3 + 4, 1 + 4]], np.uint8)  # levels 2, 3, 1 with b = 3
    xh = oracle.reconstruct(sym, (1, 1, 1, 3), T, mu, 1.0, 3)
    assert xh.reshape(-1).tolist() == [11.0, 22.0, 33.0]


def test_layouts_agree(oracle):
    s = synth.FeatureMapStream(C=8, H=3, W=5, rank=2, seed=1)
    x = s.images(2)
    T, mu, _, A = oracle.fit(x)
    T2, mu2, _, A2 = oracle.fit(synth.to_layout(x, synth.NCHW), synth.NCHW)
    assert (T == T2).all() and (mu == mu2).all() and A == A2
    y1 = oracle.project(x, T, mu)
    y2 = oracle.project(synth.to_layout(x, synth.NCHW), T, mu, synth.NCHW)
    assert (y1 == y2).all()
    sym = oracle.quantize(y1, oracle.delta(A, 5), 5)
    xh1 = oracle.reconstruct(sym, x.shape, T, mu, oracle.delta(A, 5), 5)
    xh2 = oracle.reconstruct(sym, (2, 8, 3, 5), T, mu, oracle.delta(A, 5), 5, synth.NCHW)
    assert (np.transpose(xh2, (0, 2, 3, 1)) == xh1).all()


def test_quantizer_hand_cases(oracle):
    """Round half to even, mid-tread, clamp to [-2^(b-1), 2^(b-1)-1], symbol = level + 2^(b-1)."""
    y = np.array([0.5, 1.5, 2.5, -0.5, -1.5, 0.49, -0.51, 0.0, 100.0, -100.0, 3.49, 3.51, -4.5, -4.51])
    sym, margin = oracle.quantize(y, 1.0, 3, want_margin=True)
    lev = sym.astype(int) - 4
    assert lev.tolist() == [0, 2, 2, 0, -2, 0, -1, 0, 3, -4, 3, 3, -4, -4]
    assert np.allclose(margin[:5], 0) and margin[5] == pytest.approx(0.01) and margin[7] == pytest.approx(0.5)
    assert (oracle.quantize(np.array([-9.0, -1.2, 0.2, 9.0]), 1.0, 2).astype(int) - 2).tolist() == [-2, -1, 0, 1]
    # the step scales the grid
    assert (oracle.quantize(np.array([0.26, -0.74]), 0.5, 4).astype(int) - 8).tolist() == [1, -1]


def test_delta_from_range(oracle):
    assert oracle.delta(127.0, 8) == np.float32(1.0)
    assert oracle.delta(3.0, 2) == np.float32(3.0)
    assert oracle.delta(1.0, 4) == np.float32(1.0 / 7.0)
    assert oracle.delta(0.0, 4) == np.float32(1.0)


def test_identity_basis_is_plain_quantization(oracle):
    rng = np.random.default_rng(3)
    x = rng.uniform(-3, 3, (1, 7, 7, 5)).astype(np.float32)
    T = np.eye(5, dtype=np.float32)
    mu = np.zeros(5, np.float32)
    sym = oracle.quantize(oracle.project(x, T, mu), 0.25, 6)
    expect = np.clip(np.rint(x.reshape(-1, 5).astype(np.float64) / 0.25), -32, 31) + 32
    assert (sym == expect).all()


def test_parseval_and_high_rate_distortion(oracle):
    """||x - x_hat|| = ||y - y_hat|| for an orthonormal T; without clipping D ~ Delta^2/12 (section 3, appendix D)."""
    s = synth.FeatureMapStream(C=16, H=32, W=32, rank=16, act="none", seed=11)
    x = s.images(4)
    T, mu, eig, A = oracle.fit(x)
    bits = 8
    d = oracle.delta(A, bits)
    y = oracle.project(x, T, mu)
    sym = oracle.quantize(y, d, bits)
    yh = float(d) * (sym.astype(np.float64) - 128)
    xh = oracle.reconstruct(sym, x.shape, T, mu, d, bits)
    ex = np.linalg.norm(x.astype(np.float64) - xh)
    ey = np.linalg.norm(y - yh)
    assert ex == pytest.approx(ey, rel=1e-5)
    D = oracle.mse(x, xh)
    assert D == pytest.approx(float(d) ** 2 / 12, rel=0.05)
    assert D == pytest.approx(((x.astype(np.float64) - xh) ** 2).mean(), rel=1e-12)


def test_gaussian_rate_matches_high_rate_theory(oracle):
    """iid N(0, sigma^2), T = I: H ~ log2(sqrt(2 pi e) sigma / Delta) for Delta well below sigma
    (appendix D: D_i ~ (pi e / 6) sigma_i^2 2^(-2 R_i) combined with D = Delta^2 / 12)."""
    rng = np.random.default_rng(13)
    sigma, d = 1.7, 0.2
    y = rng.standard_normal(400000) * sigma
    sym = oracle.quantize(y, d, 8)
    H = oracle.entropy(oracle.histogram(sym, 8))
    assert H == pytest.approx(np.log2(np.sqrt(2 * np.pi * np.e) * sigma / d), abs=0.05)


def test_transform_coding_ordering(oracle):
    """On correlated maps: bits/value of PCA+Q+VLC < Q+VLC < b (section 4 ablation), and
    low-variance components collapse onto the zero level (appendix 'Projection into principal components')."""
    s = synth.FeatureMapStream(C=32, H=28, W=28, rank=8, act="relu", seed=2)
    x = s.images(4)
    bits = 6
    T, mu, eig, A = oracle.fit(x)
    d = oracle.delta(A, bits)
    sym = oracle.quantize(oracle.project(x, T, mu), d, bits)
    h = oracle.histogram(sym, bits)
    ln = oracle.huffman_lengths(h[:64])
    R_pca = float((h[:64] * ln).sum()) / sym.size
    # direct quantization with the same step on the raw (mean-removed) activations
    I = np.eye(32, dtype=np.float32)
    sym_q = oracle.quantize(oracle.project(x, I, mu), d, bits)
    hq = oracle.histogram(sym_q, bits)
    lq = oracle.huffman_lengths(hq[:64])
    R_q = float((hq[:64] * lq).sum()) / sym_q.size
    assert R_pca < R_q < bits
    # at a coarse step the last component maps to a single value (the zero level)
    sym4 = oracle.quantize(oracle.project(x, T, mu), oracle.delta(A, 4), 4)
    assert (sym4[:, -1] == 8).mean() > 0.99 and (sym4[:, 0] == 8).mean() < 0.5
    # same step => same distortion to first order, so the rate gain is not bought with error
    xh = oracle.reconstruct(sym, x.shape, T, mu, d, bits)
    xq = oracle.reconstruct(sym_q, x.shape, I, mu, d, bits)
    assert oracle.mse(x, xh) <= 1.2 * oracle.mse(x, xq)
