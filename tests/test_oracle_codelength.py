"""Pins for the oracle's code-length accounting (Thm 5.3 and its proof in App. C.1; Huffman coding, App. C.3):
index counts against numpy, Huffman totals against textbook cases and the entropy sandwich H <= L < H + 1,
the expected number of non-zeros (lemma in App. C.1) by Monte Carlo, and the report's arithmetic by hand."""
import numpy as np
import pytest


def uniform_levels(S):
    return (np.arange(S, dtype=np.float64) / (S - 1)).astype(np.float32)


def test_huffman_totals(oracle):
    assert oracle.huffman_bits([8, 4, 2, 2]) == 8 * 1 + 4 * 2 + 2 * 3 + 2 * 3             # dyadic: equals n H = 28
    assert oracle.huffman_bits([25, 25, 20, 15, 15]) == 230                              # textbook: 2.3 bits / symbol
    assert oracle.huffman_bits([5] * 8) == 5 * 8 * 3                                     # uniform over 2^3 symbols
    assert oracle.huffman_bits([0, 7, 0]) == 7                                           # one used symbol: one bit each
    assert oracle.huffman_bits([3, 0, 9]) == 12 and oracle.huffman_bits([0, 0]) == 0
    rng = np.random.default_rng(0)
    for _ in range(50):
        c = rng.integers(0, 1000, rng.integers(2, 40)).astype(np.uint64)
        c[rng.integers(0, c.size)] += 1
        n = float(c.sum())
        p = c[c > 0] / n
        H = float(-(p * np.log2(p)).sum())
        L = oracle.huffman_bits(c) / n
        assert H - 1e-12 <= L < H + 1 or np.count_nonzero(c) == 1


def test_index_counts_match_the_unpacked_codes(oracle):
    sizes, S, types = [5000, 300, 0, 20000], [8, 4, 8, 8], [0, 1, 0, 0]
    rng = np.random.default_rng(1)
    g = [rng.standard_t(3, s).astype(np.float32) for s in sizes]
    lev = [uniform_levels(s) for s in S]
    for scope in (0, 1, 2):
        msg, _, _, _ = oracle.quantize(sizes, S, lev, g, 3, 1, 0, scope=scope)
        counts = oracle.index_counts(sizes, S, types, 2, [msg, msg], scope=scope)
        _, body = oracle.layout(sizes, S, scope)
        want = np.zeros((2, 256), np.uint64)
        for l, s in enumerate(sizes):
            if s == 0:
                continue
            nb = (s + 2047) // 2048 * oracle.octet_bytes(S[l], scope)
            idx = oracle.unpack_layer(msg[int(body[l]): int(body[l]) + nb], s, S[l], scope)[1]
            want[types[l]] += 2 * np.bincount(idx, minlength=256).astype(np.uint64)
        assert np.array_equal(counts, want) and counts.sum() == 2 * sum(sizes)


def test_expected_nonzeros_lemma(oracle):
    """E ||Q(v)||_0 = sum_m (1 - p_0^m) mu^m d with p_0 = E[(l_1 - u)/l_1 ; u < l_1] (Proposition + Lemma, App. C.1)."""
    S, d, seeds = 8, 4096, 300
    lev = np.array([0, .03, .08, .15, .3, .5, .75, 1.0], np.float32)
    v = (np.random.default_rng(2).standard_normal(d) * 0.7).astype(np.float32)
    norm = float(np.sqrt(np.sum(v.astype(np.float64) ** 2)))
    u = np.abs(v.astype(np.float64)) / norm
    p0 = float(np.mean(np.where(u < lev[1], (lev[1] - u) / lev[1], 0.0)))
    nz = []
    for seed in range(seeds):
        msg, _, _, _ = oracle.quantize([d], [S], [lev], [v], seed, 1, 0)
        c = oracle.index_counts([d], [S], [0], 1, [msg])
        nz.append(oracle.code_length([S], c, 1)["nonzeros"])
    want = (1 - p0) * d
    sd = np.sqrt(d * 0.25 / seeds)                                     # generous: Bernoulli variance <= 1/4
    assert abs(np.mean(nz) - want) < 5 * sd


def test_report_arithmetic(oracle):
    counts = np.zeros((2, 256), np.uint64)
    counts[0, :4] = [8, 4, 2, 2]          # S = 4: interior levels j = 1, 2
    counts[1, :2] = [6, 10]               # S = 2: no interior level
    r = oracle.code_length([4, 2], counts, num_norms=3)
    assert r["coordinates"] == 32 and r["nonzeros"] == 8 + 10
    assert r["fixed_bits"] == 32 * 3 + 16 * 3 + 16 * 2
    h0 = 1.75
    h1 = float(-(6 / 16) * np.log2(6 / 16) - (10 / 16) * np.log2(10 / 16))
    assert r["entropy_bits"] == pytest.approx(96 + 18 + 16 * h0 + 16 * h1, rel=1e-14)
    assert r["huffman_bits"] == 96 + 18 + 28 + 16
    h_int0 = float(-(4 / 16) * np.log2(4 / 16) - (2 / 16) * np.log2(2 / 16))
    assert r["paper_bits"] == pytest.approx(96 + (8 + 16 * (1 + h_int0)) + (10 + 16 * 1.0), rel=1e-14)
    assert r["entropy_bits"] <= r["huffman_bits"] <= r["fixed_bits"]
