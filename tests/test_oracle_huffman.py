"""Pins for the oracle's statistics, Huffman and canonical-code steps
(section 3.1 'Variable length coding'; appendix 'Huffman encoder as VLC')."""
import itertools
import json
import os

import numpy as np
import pytest

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "huffman_hand_worked.json")))


def _hist256(h):
    out = np.zeros(256, np.uint64)
    out[: len(h)] = h
    return out


@pytest.mark.parametrize("case", GOLD["lengths"], ids=lambda c: c["name"])
def test_hand_worked_lengths(oracle, case):
    h = np.array(case["hist"], np.uint64)
    ln = oracle.huffman_lengths(h)
    assert ln.tolist() == case["len"]
    assert int((h * ln).sum()) == case["total_bits"]


@pytest.mark.parametrize("case", GOLD["canonical"], ids=lambda c: c["name"])
def test_hand_worked_canonical(oracle, case):
    code = oracle.canonical_codes(np.array(case["len"], np.uint8))
    assert code.tolist() == case["code"]


def test_histogram_brute_force(oracle):
    rng = np.random.default_rng(1)
    for bits in (2, 5, 8):
        s = rng.integers(0, 1 << bits, 1000).astype(np.uint8)
        h = oracle.histogram(s, bits)
        assert h.sum() == s.size
        assert h.tolist() == np.bincount(s, minlength=256).tolist()
    with pytest.raises(oracle.OracleError):
        oracle.histogram(np.array([4], np.uint8), 2)  # symbol outside the 2-bit alphabet


def test_entropy_closed_forms(oracle):
    assert oracle.entropy(np.array([4, 4, 4, 4], np.uint64)) == pytest.approx(2.0, abs=1e-12)
    assert oracle.entropy(np.array([1, 1, 2, 4], np.uint64)) == pytest.approx(1.75, abs=1e-12)
    assert oracle.entropy(np.array([0, 9, 0], np.uint64)) == 0.0
    p = np.array([3, 5, 11, 2], np.float64) / 21
    assert oracle.entropy(np.array([3, 5, 11, 2], np.uint64)) == pytest.approx(-(p * np.log2(p)).sum(), abs=1e-12)


def _kraft(ln):
    return sum(2.0 ** -int(l) for l in ln if l)


def test_kraft_equality_and_rate_bound(oracle):
    """Any Huffman code is complete (Kraft sum 1) and H <= R < H + 1."""
    rng = np.random.default_rng(2)
    for trial in range(200):
        K = int(rng.choice([4, 16, 64, 256]))
        used = int(rng.integers(2, K + 1))
        h = np.zeros(K, np.uint64)
        idx = rng.choice(K, used, replace=False)
        scale = float(rng.choice([3, 100, 1e6]))
        h[idx] = np.maximum(1, (rng.pareto(1.0, used) * scale).astype(np.uint64))
        ln = oracle.huffman_lengths(h)
        assert ((ln > 0) == (h > 0)).all()
        assert _kraft(ln) == 1.0
        V = float(h.sum())
        R = float((h * ln).sum()) / V
        H = oracle.entropy(h)
        assert H - 1e-12 <= R < H + 1.0


def _all_length_vectors(n, maxlen):
    """Every length vector of n symbols with Kraft sum <= 1 (the prefix-code existence condition)."""
    for ln in itertools.product(range(1, maxlen + 1), repeat=n):
        if sum(2.0 ** -l for l in ln) <= 1.0:
            yield ln


def test_optimal_by_brute_force(oracle):
    """Total cost equals the minimum over every feasible length vector (<= 6 symbols)."""
    rng = np.random.default_rng(3)
    for n in (2, 3, 4, 5, 6):
        vecs = list(_all_length_vectors(n, n))  # an optimal code over n symbols never exceeds depth n-1
        for trial in range(12):
            h = rng.integers(1, 30, n).astype(np.uint64)
            best = min(sum(int(a) * b for a, b in zip(h, v)) for v in vecs)
            ln = oracle.huffman_lengths(h)
            assert int((h * ln).sum()) == best, (h, ln)


def test_fibonacci_depth_bound(oracle):
    """Fibonacci counts give the deepest tree a total count allows: depth n-1 for n leaves."""
    fib = [1, 1]
    while len(fib) < 40:
        fib.append(fib[-1] + fib[-2])
    h = np.array(fib, np.uint64)
    ln = oracle.huffman_lengths(h)
    assert ln.max() == 39
    assert ln.tolist() == [39, 39] + list(range(38, 0, -1))
    assert _kraft(ln) == 1.0


def test_canonical_codes_are_prefix_free_and_ordered(oracle):
    rng = np.random.default_rng(4)
    for trial in range(50):
        K = int(rng.choice([4, 16, 256]))
        h = rng.integers(0, 1000, K).astype(np.uint64) ** 2
        if (h > 0).sum() < 2:
            continue
        ln = oracle.huffman_lengths(h)
        code = oracle.canonical_codes(ln)
        words = sorted((format(int(code[s]), "b").zfill(int(ln[s])), s) for s in range(K) if ln[s])
        for (a, _), (b, _) in zip(words, words[1:]):
            assert not b.startswith(a)
        order = sorted((int(ln[s]), s) for s in range(K) if ln[s])
        vals = [int(code[s]) << (int(ln.max()) - l) for l, s in order]
        assert vals == sorted(vals) and len(set(vals)) == len(vals)
        assert vals[0] == 0


def test_invalid_inputs(oracle):
    with pytest.raises(oracle.OracleError):
        oracle.huffman_lengths(np.zeros(16, np.uint64))  # nothing to code
