"""Pins for the oracle's truncated projection / reconstruction (section 4 'Ablation study': the least
significant principal components are dropped) and for its calibration over several tensors (section 3.1
'Linear transform': the covariance of a small batch, which may be updated online)."""
import numpy as np
import pytest

from paper_1905_10830_amd import synth


def _nhwc(points):
    a = np.asarray(points, np.float32)
    return a.reshape(1, a.shape[0], 1, a.shape[1])


def test_keep_all_is_the_untruncated_path(oracle):
    s = synth.FeatureMapStream(C=12, H=6, W=6, rank=5, act="relu", seed=2)
    x = s.images(2)
    T, mu, eig, A = oracle.fit(x)
    y = oracle.project(x, T, mu)
    assert np.array_equal(oracle.project_keep(x, T, mu, 12), y)
    d = oracle.delta(A, 6)
    sym = oracle.quantize(y, d, 6)
    assert np.array_equal(oracle.reconstruct_keep(sym, x.shape, T, mu, d, 6, 12), oracle.reconstruct(sym, x.shape, T, mu, d, 6))


def test_two_channel_hand_case(oracle):
    """T = 45-degree rotation, mu = 0, keep 1: y = ((a+b)/sqrt2, 0) and x_hat = ((a+b)/2, (a+b)/2)."""
    r = 1 / np.sqrt(2)
    T = np.array([[r, r], [r, -r]], np.float32)
    mu = np.zeros(2, np.float32)
    x = _nhwc([(3.0, 1.0), (-2.0, 5.0)])
    y = oracle.project_keep(x, T, mu, 1)
    assert np.allclose(y, [[4 * r, 0], [3 * r, 0]], atol=1e-6)
    assert (y[:, 1] == 0).all()
    # symbols on an exact grid: Delta = r/4 makes y0/Delta = 16 and 12
    d = np.float32(r / 4)
    sym = oracle.quantize(y, d, 8)
    assert sym.tolist() == [[128 + 16, 128], [128 + 12, 128]]
    xh = oracle.reconstruct_keep(sym, x.shape, T, mu, d, 8, 1).reshape(2, 2)
    assert np.allclose(xh, [[2, 2], [1.5, 1.5]], atol=1e-6)


def test_truncation_error_is_the_sum_of_the_dropped_eigenvalues(oracle):
    """PCA: on the data the basis was fitted on, dropping components k >= keep leaves a mean squared error per
    pixel of sum_{k >= keep} lambda_k (no quantizer)."""
    s = synth.FeatureMapStream(C=16, H=10, W=10, rank=6, act="none", seed=9)
    x = s.images(4)
    T, mu, eig, A = oracle.fit(x)
    flat = x.reshape(-1, 16).astype(np.float64)
    for keep in (1, 5, 11, 16):
        y = oracle.project_keep(x, T, mu, keep)
        assert (y[:, keep:] == 0).all()
        xh = y @ T.astype(np.float64) + mu.astype(np.float64)
        err = ((flat - xh) ** 2).sum(axis=1).mean()
        assert err == pytest.approx(eig[keep:].sum(), rel=1e-5, abs=1e-9 * eig[0])
    # kept coefficients are the untruncated ones
    assert np.array_equal(oracle.project_keep(x, T, mu, 5)[:, :5], oracle.project(x, T, mu)[:, :5])


def test_reconstruction_ignores_the_dropped_symbols(oracle):
    s = synth.FeatureMapStream(C=10, H=5, W=7, rank=4, act="relu", seed=4)
    for layout in (synth.NHWC, synth.NCHW):
        x = synth.to_layout(s.images(2), layout)
        T, mu, eig, A = oracle.fit(x, layout)
        d = oracle.delta(A, 5)
        res = oracle.encode_keep(x, T, mu, d, 5, keep=4, layout=layout)
        sym = res["sym"]
        assert (sym[:, 4:] == 16).all()                      # the zero level 2^(b-1)
        assert np.array_equal(sym[:, :4], oracle.quantize(oracle.project(x, T, mu, layout), d, 5)[:, :4])
        want = oracle.reconstruct(sym, x.shape, T, mu, d, 5, layout)   # zero-level symbols contribute nothing
        junk = sym.copy()
        junk[:, 4:] = np.random.default_rng(0).integers(0, 32, size=junk[:, 4:].shape)
        got = oracle.reconstruct_keep(junk, x.shape, T, mu, d, 5, 4, layout)
        assert np.abs(got - want).max() < 1e-12
        # the container decodes to the same symbols
        xh, sym2 = oracle.decode(res["stream"], x.shape, T, mu, 5, layout)
        assert np.array_equal(sym2, sym)


def test_truncation_lowers_the_rate_and_raises_the_error(oracle):
    s = synth.FeatureMapStream(C=32, H=8, W=8, rank=8, act="relu", seed=6)
    x = s.images(4)
    T, mu, eig, A = oracle.fit(x)
    d = oracle.delta(A, 6)
    last_h, last_e = None, None
    for keep in (32, 16, 4):
        res = oracle.encode_keep(x, T, mu, d, 6, keep)
        h = oracle.entropy(res["hist"])
        e = oracle.mse(x, oracle.reconstruct_keep(res["sym"], x.shape, T, mu, d, 6, keep))
        if last_h is not None:
            assert h <= last_h + 1e-12 and e >= last_e - 1e-12
        last_h, last_e = h, e


def test_dynamic_range_hand_case(oracle):
    r = 1 / np.sqrt(2)
    A = oracle.dynamic_range(_nhwc([(2.0, 0.0), (-1.0, -4.0), (0.5, 0.5)]), [r, r], [0.0, 0.0])
    assert A == pytest.approx(5 * r, rel=1e-6)
    A = oracle.dynamic_range(_nhwc([(2.0, 0.0)]), [1.0, 0.0], [0.5, 9.0])
    assert A == pytest.approx(1.5, rel=1e-6)


@pytest.mark.parametrize("layout", [synth.NHWC, synth.NCHW])
def test_fit_of_one_tensor_is_the_plain_fit(oracle, layout):
    s = synth.FeatureMapStream(C=9, H=6, W=5, rank=4, act="relu", seed=3)
    x = synth.to_layout(s.images(3), layout)
    T, mu, eig, A = oracle.fit(x, layout)
    T2, mu2, eig2, A2 = oracle.fit_online([x], x, layout)
    assert np.array_equal(T, T2) and np.array_equal(mu, mu2) and np.array_equal(eig, eig2) and A == A2


def test_fit_over_several_tensors_is_the_fit_of_their_union(oracle):
    s = synth.FeatureMapStream(C=14, H=7, W=9, rank=5, act="relu", seed=8)
    imgs = s.images(7)
    parts = [imgs[:1], imgs[1:4], imgs[4:]]
    T, mu, eig, A = oracle.fit_online(parts, parts[-1])
    flat = imgs.reshape(-1, 14).astype(np.float64)
    assert np.allclose(mu, flat.mean(0), atol=1e-6)
    w = np.linalg.eigvalsh(np.cov(flat.T, bias=True))[::-1]
    assert np.allclose(eig, w, rtol=1e-9, atol=1e-12 * w[0])
    # the range is that of the last tensor, not of the union
    y0 = (parts[-1].reshape(-1, 14).astype(np.float64) - mu.astype(np.float64)) @ T[0].astype(np.float64)
    assert A == pytest.approx(np.abs(y0).max(), rel=1e-6)
    # order of the tensors does not matter (up to rounding)
    T3, mu3, eig3, _ = oracle.fit_online(parts[::-1], parts[-1])
    assert np.allclose(eig3, eig, rtol=1e-12) and np.allclose(mu3, mu)
