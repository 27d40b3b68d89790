"""Pins for the oracle's scalar building blocks: exact-comparison square root / reciprocal, the canonical
fp64 sum of squares, and the counter-based generator (its published known-answer vectors, plus statistical pins
on the way the draws are indexed)."""
import math
from fractions import Fraction

import numpy as np
import pytest


def _next_up(x: np.float32) -> np.float32:
    return (np.array([x], dtype=np.float32).view(np.uint32) + np.uint32(1)).view(np.float32)[0]


def test_sqrt_floor_is_the_largest_float_whose_square_fits(oracle):
    rng = np.random.default_rng(1)
    vals = list(np.exp(rng.uniform(-80, 80, 400))) + [0.0, 1.0, 4.0, 2.0, 1e-60, 3.0e76, float(np.float32(3.4e38)) ** 2]
    for s in vals:
        n = oracle.sqrt_floor(s)
        assert Fraction(float(n)) ** 2 <= Fraction(s)
        if n < np.finfo(np.float32).max:
            assert Fraction(float(_next_up(n))) ** 2 > Fraction(s)
        if s > 1e-70:
            assert abs(float(n) - math.sqrt(s)) <= float(np.spacing(np.float32(math.sqrt(s))))
    # exact squares are recovered exactly
    for v in [1.0, 3.0, 0.15625, 1234.5, 2.0 ** -60]:
        assert float(oracle.sqrt_floor(v * v)) == v
    # not-a-number / infinity / negative: 0 (the caller raises the non-finite flag)
    for bad in [float("nan"), float("inf"), -1.0]:
        assert float(oracle.sqrt_floor(bad)) == 0.0


def test_rcp_floor_is_the_largest_float_with_product_at_most_one(oracle):
    rng = np.random.default_rng(2)
    xs = np.exp(rng.uniform(-60, 60, 400)).astype(np.float32)
    for x in list(xs) + [np.float32(1.0), np.float32(3.0), np.float32(0.1), np.float32(2.0 ** -100)]:
        r = oracle.rcp_floor(x)
        assert Fraction(float(x)) * Fraction(float(r)) <= 1
        assert Fraction(float(x)) * Fraction(float(_next_up(r))) > 1
        assert abs(float(r) * float(x) - 1.0) < 3e-7
    for p in [-3, 0, 5, 20]:
        assert float(oracle.rcp_floor(np.float32(2.0 ** p))) == 2.0 ** -p
    assert float(oracle.rcp_floor(0.0)) == 0.0
    assert float(oracle.rcp_floor(float("inf"))) == 0.0
    assert float(oracle.rcp_floor(-2.0)) == 0.0


@pytest.mark.parametrize("n", [0, 1, 3, 255, 256, 257, 4099, 16384, 16385, 70001, 16384 * 257 + 5])
def test_sumsq_equals_the_exact_sum_within_fp64_rounding(oracle, n):
    rng = np.random.default_rng(n)
    v = (rng.standard_normal(n) * np.exp(rng.uniform(-10, 10, n))).astype(np.float32)
    s = oracle.sumsq(v)
    exact = math.fsum((v.astype(np.float64) ** 2).tolist())
    assert abs(s - exact) <= 1e-13 * exact + 0.0
    if n:
        nrm = oracle.sqrt_floor(s)
        ref = math.sqrt(exact)
        assert abs(float(nrm) - ref) <= float(np.spacing(np.float32(ref)))


def test_sumsq_of_exactly_representable_squares_is_exact(oracle):
    # small integers: every partial sum is exact in fp64 whatever the order, so the result is the integer sum
    rng = np.random.default_rng(7)
    v = rng.integers(-1000, 1000, 50000).astype(np.float32)
    assert oracle.sumsq(v) == float(np.sum(v.astype(np.int64) ** 2))


def test_sumsq_detects_a_dropped_or_doubled_element(oracle):
    v = np.zeros(20000, dtype=np.float32)
    for pos in [0, 3, 255, 256, 4095, 16383, 16384, 19999]:
        w = v.copy()
        w[pos] = 3.0
        assert oracle.sumsq(w) == 9.0


# ---------------------------------------------------------------- generator: statistical pins
def _outputs(oracle, n, key=(1, 0), ctr_hi=(0, 1, 0)):
    out = np.zeros((n, 4), dtype=np.uint32)
    for i in range(n):
        out[i] = oracle.philox4x32_10([i, *ctr_hi], key)
    return out


def test_generator_known_answer_vectors(oracle):
    """Philox4x32-10 against the published known-answer vectors (tests/golden/philox4x32_10_kat.txt)."""
    import os

    path = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")
    rows = [ln.split() for ln in open(path) if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        v = [int(x, 16) for x in r]
        assert [int(x) for x in oracle.philox4x32_10(v[0:4], v[4:6])] == v[6:10]


def test_generator_words_are_uniform_and_balanced(oracle):
    out = _outputs(oracle, 20000).reshape(-1)
    # every bit position is set about half the time
    bits = ((out[:, None] >> np.arange(32, dtype=np.uint32)) & 1).mean(axis=0)
    assert np.all(np.abs(bits - 0.5) < 5 * 0.5 / math.sqrt(out.size))
    # chi-square on the top byte and on the low byte
    for shift in (24, 0):
        cnt = np.bincount(((out >> shift) & 0xFF).astype(np.int64), minlength=256)
        chi2 = ((cnt - out.size / 256) ** 2 / (out.size / 256)).sum()
        assert chi2 < 255 + 6 * math.sqrt(2 * 255)


def test_generator_avalanche_and_injectivity(oracle):
    base = oracle.philox4x32_10([5, 6, 7, 8], [9, 10])
    flips = []
    for word in range(4):
        for bit in (0, 7, 16, 31):
            c = [5, 6, 7, 8]
            c[word] ^= 1 << bit
            o = oracle.philox4x32_10(c, [9, 10])
            flips.append(sum(bin(int(a) ^ int(b)).count("1") for a, b in zip(o, base)))
    for word in range(2):
        k = [9, 10]
        k[word] ^= 1 << 3
        o = oracle.philox4x32_10([5, 6, 7, 8], k)
        flips.append(sum(bin(int(a) ^ int(b)).count("1") for a, b in zip(o, base)))
    assert all(35 < f < 93 for f in flips), flips      # 128 output bits, about half flip
    # a keyed bijection of the counter: distinct counters give distinct outputs
    out = _outputs(oracle, 5000)
    assert len({tuple(r) for r in out.tolist()}) == 5000


def test_draws_of_neighbouring_coordinates_are_uncorrelated(oracle):
    n = 1 << 15
    w = np.array([oracle.draw16(1, 1, 0, 0, e) for e in range(n)], dtype=np.float64)
    assert w.min() >= 0 and w.max() <= 65535
    u = (w + 0.5) / 65536
    assert abs(u.mean() - 0.5) < 5 / math.sqrt(12 * n)
    for lag in (1, 2, 3, 4, 8, 256, 512):
        r = np.corrcoef(u[:-lag], u[lag:])[0, 1]
        assert abs(r) < 5 / math.sqrt(n), (lag, r)
    cnt = np.bincount((w // 256).astype(np.int64), minlength=256)
    chi2 = ((cnt - n / 256) ** 2 / (n / 256)).sum()
    assert chi2 < 255 + 6 * math.sqrt(2 * 255)


def test_draw_depends_on_every_index(oracle):
    base = [oracle.draw16(1, 1, 0, 0, e) for e in range(2048)]
    for kw in [dict(seed=2), dict(round_=2), dict(node=1), dict(layer=1), dict(seed=1 + (1 << 32))]:
        a = dict(seed=1, round_=1, node=0, layer=0)
        a.update(kw)
        other = [oracle.draw16(a["seed"], a["round_"], a["node"], a["layer"], e) for e in range(2048)]
        same = sum(int(x == y) for x, y in zip(base, other))
        assert same < 10, (kw, same)
    # the eight coordinates served by one generator call all get different 16-bit fields
    out = oracle.philox4x32_10([(3 << 6) | 5, 0, 1, 0], [1, 0])
    es = [3 * 512 + 4 * 5 + j for j in range(4)] + [3 * 512 + 256 + 4 * 5 + j for j in range(4)]
    got = [oracle.draw16(1, 1, 0, 0, e) for e in es]
    want = [int(out[j]) & 0xFFFF for j in range(4)] + [int(out[j]) >> 16 for j in range(4)]
    assert got == want
