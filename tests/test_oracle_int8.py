"""Pins for the oracle's 8-bit path (section 3.1 'Linear transform': the PCA matrix stored at 8 bits;
section 5: 8-bit activations): hand cases, brute force in Python integers, and agreement with the pinned
floating-point oracle run on the dequantized basis and activations."""
import math
from fractions import Fraction

import numpy as np
import pytest

from paper_1905_10830_amd import synth


def _rne(fr):
    """Round a Fraction half to even."""
    f = math.floor(fr)
    d = fr - f
    if d > Fraction(1, 2) or (d == Fraction(1, 2) and f % 2 == 1):
        return f + 1
    return f


def test_basis8_hand_case(oracle):
    T = np.array([[0.6, 0.8], [-0.8, 0.6]], np.float32)
    mu = np.array([1.0, 0.26], np.float32)
    Tq, sT, mf = oracle.basis8(T, mu, act_scale=0.5)
    assert sT == np.float32(np.float64(np.float32(0.8)) / 127.0)
    # 0.6 / (0.8 / 127) = 95.25, 0.8 -> 127
    assert Tq.tolist() == [[95, 127], [-127, 95]]
    # mean on the activations' grid with 8 fraction bits: 1.0 / 0.5 * 256 = 512, 0.26 / 0.5 * 256 = 133.12
    assert mf.tolist() == [512, 133]


def test_quantize_u8_hand_case(oracle):
    """C = 2, Tq = [[100, 0], [0, -50]], mf = [256, 0] (mean 1 activation unit on channel 0), s_T = 0.01,
    s_x = 0.5, Delta = 0.25: y = s_T s_x Tq (xq - mf / 256) = 0.5 (xq0 - 1), -0.25 xq1."""
    Tq = np.array([[100, 0], [0, -50]], np.int8)
    mf = np.array([256, 0], np.int32)
    xq = np.array([[3, 2], [0, 1], [201, 255], [1, 0]], np.uint8).reshape(1, 4, 1, 2)
    sym = oracle.quantize_u8(xq, Tq, 0.01, mf, 0.5, 0.25, 6)
    # levels y / Delta: (4, -2), (-2, -1), (400 -> clamp 31, -255 -> clamp -32), (0, 0); symbol = level + 32
    assert sym.tolist() == [[36, 30], [30, 31], [63, 0], [32, 32]]
    back = oracle.reconstruct_u8(sym, xq.shape, Tq, 0.01, mf, 0.5, 0.25, 6).reshape(4, 2)
    # x_hat / s_x = s_T Delta / s_x * Tq^T q + mf / 256 = 0.5 q0 + 1, -0.25 q1:
    # (3, 0.5 -> tie -> 0), (0, 0.25 -> 0), (16.5 -> tie -> 16, 8), (1, 0)
    assert back.tolist() == [[3, 0], [0, 0], [16, 8], [1, 0]]


@pytest.mark.parametrize("layout", [synth.NHWC, synth.NCHW])
def test_u8_path_against_python_integers(oracle, layout):
    """Brute force with exact rationals for the sums; the one fp64 product / fused multiply-add per value is
    replayed with numpy's float64 and math.fma-free exact rational rounding of the same operands."""
    rng = np.random.default_rng(3)
    C, n, h, w, bits = 5, 2, 3, 2, 5
    Tq = rng.integers(-127, 128, size=(C, C)).astype(np.int8)
    mf = rng.integers(0, 40000, size=C).astype(np.int32)
    shape = (n, h, w, C) if layout == synth.NHWC else (n, C, h, w)
    xq = rng.integers(0, 256, size=shape).astype(np.uint8)
    sT, sx, d = np.float32(0.0071), np.float32(0.043), np.float32(0.9)
    sym = oracle.quantize_u8(xq, Tq, sT, mf, sx, d, bits, layout)
    px = (xq if layout == synth.NHWC else np.transpose(xq, (0, 2, 3, 1))).reshape(-1, C)
    g = (float(sT) * float(sx)) / (256.0 * float(d))            # the oracle's fp64 factor, same expression
    half = 1 << (bits - 1)
    for p in range(px.shape[0]):
        for k in range(C):
            num = 256 * sum(int(Tq[k, c]) * int(px[p, c]) for c in range(C)) - sum(int(Tq[k, c]) * int(mf[c]) for c in range(C))
            t = Fraction(num) * Fraction(g)                          # exact product of the two fp64 operands
            lv = _rne(Fraction(float(t)))                            # correctly rounded to fp64, then to integer
            lv = max(-half, min(half - 1, lv))
            assert sym[p, k] == lv + half, (p, k)
    out = oracle.reconstruct_u8(sym, shape, Tq, sT, mf, sx, d, bits, layout)
    opx = (out if layout == synth.NHWC else np.transpose(out, (0, 2, 3, 1))).reshape(-1, C)
    hfac = (float(sT) * float(d) * 256.0) / float(sx)
    for p in range(px.shape[0]):
        for c in range(C):
            m = sum(int(Tq[k, c]) * (int(sym[p, k]) - half) for k in range(C))
            v = float(Fraction(m) * Fraction(hfac) + Fraction(int(mf[c])))   # fused: one rounding of the exact value
            r = _rne(Fraction(v / 256.0))
            assert opx[p, c] == max(0, min(255, r)), (p, c)


def test_u8_path_agrees_with_the_float_oracle_on_dequantized_inputs(oracle):
    """Same method, other arithmetic: the float oracle on x = s_x xq with T' = s_T Tq and mu' = s_x mf / 256 must
    give the same symbols except where y / Delta sits on a rounding boundary (T' is rounded to fp32 there), and
    its reconstruction divided by s_x must round to the same 8-bit values except at ties."""
    s = synth.FeatureMapStream(C=24, H=9, W=9, rank=6, act="relu", seed=31)
    x = s.images(3)
    sx = np.float32(x.max() / 255.0)
    xq = np.clip(np.rint(x / sx), 0, 255).astype(np.uint8)
    T, mu, eig, A = oracle.fit((xq.astype(np.float32) * sx))
    bits = 6
    d = oracle.delta(A, bits)
    Tq, sT, mf = oracle.basis8(T, mu, sx)
    sym = oracle.quantize_u8(xq, Tq, sT, mf, sx, d, bits)
    Tp = (Tq.astype(np.float64) * float(sT)).astype(np.float32)
    mup = (mf.astype(np.float64) * float(sx) / 256.0).astype(np.float32)
    y = oracle.project(xq.astype(np.float32) * sx, Tp, mup)
    ref, margin = oracle.quantize(y, d, bits, want_margin=True)
    diff = sym != ref
    assert diff.mean() < 1e-3 and (not diff.any() or margin[diff].max() < 1e-4)
    back = oracle.reconstruct_u8(sym, xq.shape, Tq, sT, mf, sx, d, bits)
    xf = oracle.reconstruct(sym, xq.shape, Tp, mup, d, bits) / float(sx)
    assert np.abs(back.astype(np.float64) - np.clip(xf, 0, 255)).max() <= 0.5 + 1e-4
    # and the whole thing is a usable codec: error of the order of the quantizer's
    err = ((back.astype(np.float64) - xq) * float(sx)) ** 2
    assert err.mean() < 2.0 * float(d) ** 2 / 12 + (float(sx) ** 2) / 12 + 24 * (float(sT) * A / 2) ** 2 / 12


def test_u8_symbols_do_not_depend_on_layout(oracle):
    s = synth.FeatureMapStream(C=7, H=4, W=5, rank=3, act="relu", seed=2)
    x = s.images(2)
    sx = np.float32(x.max() / 255.0)
    xq = np.clip(np.rint(x / sx), 0, 255).astype(np.uint8)
    T, mu, eig, A = oracle.fit(xq.astype(np.float32) * sx)
    Tq, sT, mf = oracle.basis8(T, mu, sx)
    d = oracle.delta(A, 4)
    a = oracle.quantize_u8(xq, Tq, sT, mf, sx, d, 4, synth.NHWC)
    b = oracle.quantize_u8(synth.to_layout(xq, synth.NCHW), Tq, sT, mf, sx, d, 4, synth.NCHW)
    assert np.array_equal(a, b)
    ra = oracle.reconstruct_u8(a, xq.shape, Tq, sT, mf, sx, d, 4, synth.NHWC)
    rb = oracle.reconstruct_u8(a, synth.to_layout(xq, synth.NCHW).shape, Tq, sT, mf, sx, d, 4, synth.NCHW)
    assert np.array_equal(synth.to_layout(ra, synth.NCHW), rb)
