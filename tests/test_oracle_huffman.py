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


# ---- code table fixed at calibration time (section 3.1 leaves open when the Huffman table is made) ----
def test_static_table_hand_worked(oracle):
    # counts 7,1,0,0 -> smoothed 8,2,1,1: merge 1+1, then 2+2, then 4+8 -> depths 1,2,3,3
    assert oracle.static_lengths(np.array([7, 1, 0, 0], np.uint64)).tolist() == [1, 2, 3, 3]
    # all counts equal (here: no calibration data at all): a fixed-length code
    assert oracle.static_lengths(np.zeros(16, np.uint64)).tolist() == [4] * 16
    # smoothing changes nothing where one more count per symbol cannot reorder the merges
    assert oracle.static_lengths(np.array([80, 40, 20, 10], np.uint64)).tolist() == \
        oracle.huffman_lengths(np.array([80, 40, 20, 10], np.uint64)).tolist() == [1, 2, 3, 3]


def test_static_table_is_complete_and_ordered(oracle):
    rng = np.random.default_rng(31)
    for bits in (2, 4, 6, 8):
        K = 1 << bits
        h = np.zeros(K, np.uint64)
        used = rng.choice(K, size=max(2, K // 3), replace=False)
        h[used] = rng.geometric(0.002, used.size)
        ln = oracle.static_lengths(h)
        assert ln.min() >= 1                                          # every symbol of the alphabet has a code
        assert sum(2.0 ** -int(l) for l in ln) == 1.0                 # Kraft equality: a complete prefix code
        order = np.argsort(h, kind="stable")
        assert all(ln[order[i]] >= ln[order[i + 1]] for i in range(K - 1))  # rarer symbols never get shorter codes
        # the symbols calibration never saw share the longest lengths
        assert ln[h == 0].min() >= ln[h > 0].max()


def test_static_table_rate_bounds(oracle):
    """Coding a tensor with a table made from another sample of the same source costs at least the tensor's own
    Huffman code (optimality) and at most cross-entropy + 1 bit per symbol (Kraft: len <= -log2 q + 1 fails for
    Huffman in general, but the average obeys sum p len < H(p, q) + 1 only for Shannon lengths; so the pin is
    against the table's own source: its average length on the calibration distribution is below H + 1)."""
    rng = np.random.default_rng(32)
    bits = 6
    p = rng.dirichlet(np.full(64, 0.3))
    cal = np.bincount(rng.choice(64, 200000, p=p), minlength=64).astype(np.uint64)
    dat = np.bincount(rng.choice(64, 50000, p=p), minlength=64).astype(np.uint64)
    ls = oracle.static_lengths(cal)
    la = oracle.huffman_lengths(dat)
    assert int((dat * ls).sum()) >= int((dat * la).sum())
    q = (cal + 1) / float((cal + 1).sum())
    assert float((q * ls).sum()) < float(-(q * np.log2(q)).sum()) + 1.0
    # and the penalty on fresh data from the same source is small (a fraction of a bit per symbol)
    assert (int((dat * ls).sum()) - int((dat * la).sum())) / dat.sum() < 0.05


def test_static_table_stream_round_trip(oracle):
    rng = np.random.default_rng(33)
    bits, C, P = 4, 24, 500
    cal = np.bincount(rng.choice(16, 5000, p=rng.dirichlet(np.full(16, 0.4))), minlength=16).astype(np.uint64)
    ln = oracle.static_lengths(cal)
    sym = rng.integers(0, 16, (P, C)).astype(np.uint8)  # uniform: includes symbols calibration hardly saw
    stream = oracle.pack(sym, C, bits, 0.25, ln, oracle.canonical_codes(ln), cap=1 << 20)
    back, d, pbits = oracle.unpack(stream, P, C, bits)
    assert (back == sym).all() and d == np.float32(0.25)
    assert pbits == int(ln[sym].astype(np.uint64).sum())
