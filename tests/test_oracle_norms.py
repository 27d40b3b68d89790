"""Pins for the oracle's L^q normalisations other than q = 2 (Sec. 2.2: u_i = |v_i| / ||v||_q for an integer q; here
q = 1 and the limit q -> infinity): the statistics against their textbook definitions, unbiasedness and the exact
variance identity eq. (Var) through the whole encode/decode path, the variance bound of Thm 5.1 with its exponent
1/min(q, 2), and the weights ||v||_q^2 that eq. (Qada2) gives each sampled vector in the level fit."""
import math

import numpy as np
import pytest

L1, L2, LINF = 1, 2, 0


def uniform_levels(S):
    return (np.arange(S, dtype=np.float64) / (S - 1)).astype(np.float32)


def expo_levels(S, base=2.0):
    return np.array([0.0] + [base ** -(S - 2 - j) for j in range(S - 1)], dtype=np.float32)


def textbook_norm(v, kind):
    a = np.abs(v.astype(np.float64))
    return {L1: a.sum(), L2: math.sqrt(float((a * a).sum())), LINF: a.max() if a.size else 0.0}[kind]


def var_identity(v, norm, lev):
    """eq. (Var) per coordinate, in float64 from the definition."""
    u = np.minimum(np.abs(v.astype(np.float64)) / float(norm), 1.0)
    lev = lev.astype(np.float64)
    tau = np.clip(np.searchsorted(lev, u, side="right") - 1, 0, len(lev) - 2)
    return float(norm) ** 2 * (lev[tau + 1] - u) * (u - lev[tau])


def eps_Q(lev, d, q):
    """Thm 5.1 with M = 1 (ratio maximum over j >= 1 as in its proof); q = infinity enters through min(q, 2) = 2."""
    lev = lev.astype(np.float64)
    lbar = max(lev[j + 1] / lev[j] for j in range(1, len(lev) - 1)) if len(lev) > 2 else 1.0
    l1 = lev[1]
    mq = min(q, 2)
    dth = (2.0 / l1) ** mq
    e = (lbar - 1) ** 2 / (4 * lbar)
    return e + (l1 * d ** (1.0 / mq) - 1 if d >= dth else l1 ** 2 / 4 * d ** (2.0 / mq))


@pytest.mark.parametrize("d", [1, 5, 255, 4097, 16384 * 2 + 11, 100_003])
def test_statistics_equal_their_definitions(oracle, d):
    rng = np.random.default_rng(d)
    v = (rng.standard_t(3, d) * 10.0 ** rng.uniform(-3, 3)).astype(np.float32)
    s1 = oracle.norm_stat(v, L1)
    assert s1 == pytest.approx(float(np.abs(v.astype(np.float64)).sum()), rel=1e-13)
    assert oracle.norm_stat(v, LINF) == float(np.abs(v).max())
    assert oracle.norm_stat(v, L2) == oracle.sumsq(v)
    # integers add exactly in any order: the canonical order must give the exact sum
    w = rng.integers(-1000, 1000, d).astype(np.float32)
    assert oracle.norm_stat(w, L1) == float(np.abs(w.astype(np.int64)).sum())
    # the norms: one correctly rounded conversion of the statistic
    assert oracle.norm_of(s1, L1) == np.float32(s1)
    assert oracle.norm_of(oracle.norm_stat(v, LINF), LINF) == np.abs(v).max()
    assert oracle.weight_of(s1, L1) == s1 * s1 and oracle.weight_of(7.0, L2) == 7.0


def test_bucket_statistics_equal_their_definitions(oracle):
    rng = np.random.default_rng(3)
    for n in (1, 4, 77, 128):
        v = (rng.standard_normal(n) * 3).astype(np.float32)
        assert oracle.bucket_stat(v, L2) == oracle.bucket_sumsq(v)
        assert oracle.bucket_stat(v, LINF) == float(np.abs(v).max())
        assert oracle.bucket_stat(v, L1) == pytest.approx(float(np.abs(v.astype(np.float64)).sum()), rel=3e-7)
        w = rng.integers(-50, 50, n).astype(np.float32)
        assert oracle.bucket_stat(w, L1) == float(np.abs(w).sum())          # small integers: exact in fp32 too


def test_non_finite_entries_are_reported(oracle):
    lev = uniform_levels(4)
    for kind in (L1, LINF):
        for bad in (np.inf, -np.inf, np.nan):
            v = np.ones(300, np.float32)
            v[17] = bad
            for scope in (oracle.SCOPE_LAYER, oracle.SCOPE_VECTOR, oracle.SCOPE_BUCKET):
                assert oracle.quantize([300], [4], [lev], [v], 1, 1, 0, scope=scope, norm_kind=kind)[3] == 1
    big = np.full(8, 3e38, np.float32)                                         # sum of magnitudes beyond fp32
    assert oracle.quantize([8], [4], [lev], [big], 1, 1, 0, norm_kind=L1)[3] == 1
    assert oracle.quantize([8], [4], [lev], [big], 1, 1, 0, norm_kind=LINF)[3] == 0


def decode_all(oracle, sizes, S, msg, scope):
    return oracle.dequant_aggregate(sizes, [S] * len(sizes), [msg], scope=scope)


@pytest.mark.parametrize("kind", [L1, LINF])
@pytest.mark.parametrize("scope", [0, 1, 2])
def test_header_norm_and_range_of_u(oracle, kind, scope):
    """The message carries the kind's norm (textbook value within rounding), every decoded magnitude is
    norm * level, and no normalised coordinate exceeds 1."""
    rng = np.random.default_rng(10 * kind + scope)
    sizes = [700, 130, 2048 + 5]
    S = 8
    lev = expo_levels(S)
    g = [(rng.standard_t(3, s) * 0.01 * (l + 1)).astype(np.float32) for l, s in enumerate(sizes)]
    msg, ss, _, st = oracle.quantize(sizes, [S] * 3, [lev] * 3, g, 5, 1, 0, scope=scope, norm_kind=kind)
    assert st == 0
    hdr, body = oracle.layout(sizes, [S] * 3, scope)
    whole = np.concatenate(g)
    for l, s in enumerate(sizes):
        if scope == oracle.SCOPE_LAYER:
            want = textbook_norm(g[l], kind)
        elif scope == oracle.SCOPE_VECTOR:
            want = textbook_norm(whole, kind)
        else:
            want = None
        got = msg[int(hdr[l]): int(hdr[l]) + 4].view(np.float32)[0]
        if want is not None:
            assert got == pytest.approx(want, rel=2e-7)
            if kind == LINF:
                assert got == np.float32(want)
    out = decode_all(oracle, sizes, S, msg, scope)
    for l, s in enumerate(sizes):
        if scope == oracle.SCOPE_BUCKET:
            for b in range(0, s, 128):
                nb = textbook_norm(g[l][b: b + 128], kind)
                mags = np.abs(out[l][b: b + 128].astype(np.float64)) / nb
                assert np.all(np.min(np.abs(mags[:, None] - lev[None, :].astype(np.float64)), axis=1) < 1e-6)
                assert np.all(np.abs(out[l][b: b + 128]) <= nb * (1 + 1e-6))
        else:
            n = msg[int(hdr[l]): int(hdr[l]) + 4].view(np.float32)[0]
            mags = np.abs(out[l].astype(np.float64)) / float(n)
            assert np.all(np.min(np.abs(mags[:, None] - lev[None, :].astype(np.float64)), axis=1) < 1e-6)


@pytest.mark.parametrize("kind", [L1, LINF])
def test_unbiased_and_variance_identity_through_the_message(oracle, kind):
    """800 rounds (independent draws) of one small layer: the mean of the decoded vectors approaches v, and the mean
    squared error approaches eq. (Var) evaluated with ||v||_q -- which differs from the q = 2 value by a large factor,
    so a norm of the wrong kind anywhere in the path fails."""
    rng = np.random.default_rng(kind)
    d, S, R = 600, 8, 800
    v = (rng.standard_t(4, d) * 0.05).astype(np.float32)
    lev = uniform_levels(S)
    norm = float(oracle.norm_of(oracle.norm_stat(v, kind), kind))
    per = var_identity(v, norm, lev)
    acc = np.zeros(d)
    err = 0.0
    for t in range(1, R + 1):
        msg, _, _, st = oracle.quantize([d], [S], [lev], [v], 9, t, 0, norm_kind=kind)
        q = decode_all(oracle, [d], S, msg, 0)[0].astype(np.float64)
        acc += q
        err += float(np.sum((q - v) ** 2))
    mean = acc / R
    z = (mean - v) / np.sqrt(np.maximum(per, 1e-30) / R)
    assert np.abs(z[per > 0]).max() < 5.0
    assert err / R == pytest.approx(per.sum(), rel=0.03)
    other = var_identity(v, textbook_norm(v, L2), lev).sum()
    assert abs(other / per.sum() - 1) > 0.2


@pytest.mark.parametrize("q,kind", [(1, L1), (2, L2), (10 ** 9, LINF)])
def test_variance_bound_of_thm_5_1_for_each_q(oracle, q, kind):
    rng = np.random.default_rng(q % 97)
    for trial in range(60):
        d = int(rng.integers(2, 3000))
        S = int(rng.choice([3, 4, 8, 16]))
        lev = uniform_levels(S) if trial % 2 else expo_levels(S)
        shape = rng.choice(["t", "spike", "flat"])
        if shape == "t":
            v = rng.standard_t(3, d)
        elif shape == "spike":
            v = rng.standard_normal(d) * 1e-3
            v[rng.integers(0, d)] = 1.0
        else:
            v = rng.choice([-1.0, 1.0], d)
        v = v.astype(np.float32)
        norm = float(oracle.norm_of(oracle.norm_stat(v, kind), kind))
        exact = var_identity(v, norm, lev).sum()
        bound = eps_Q(lev, d, q) * float(np.sum(v.astype(np.float64) ** 2))
        assert exact <= bound * (1 + 1e-6), (trial, d, S, shape)
    # the exponent matters: a flat vector normalised by its L1 norm breaks the bound written for q = 2
    d, lev = 2000, uniform_levels(4)
    v = np.ones(d, np.float32)
    n1 = float(oracle.norm_of(oracle.norm_stat(v, L1), L1))
    assert var_identity(v, n1, lev).sum() > eps_Q(lev, d, 2) * d


@pytest.mark.parametrize("kind", [L1, LINF])
@pytest.mark.parametrize("scope", [0, 2])
def test_fit_weights_are_the_squared_norms(oracle, kind, scope):
    """Two nodes, each bucket of 128 made of one large entry and 127 equal small ones, the small ones of the two nodes
    far apart after normalisation: the pooled mass at each node's small-value bins is its number of sampled entries
    (equal for both) times ||v_k||_q^2 (eq. (Qada2), weights lambda_z), up to the integer scaling."""
    d, S = 1024, 8

    def make(top, small):
        v = np.full(d, small, np.float32)
        v[::128] = top
        return v

    a, b = make(1.0, 0.25), make(2.0, 0.002)
    lev = uniform_levels(S)
    levs, hist, pooled, st = oracle.fit_levels([d], [0], [S], 2, [a, b], [lev], scope=scope, norm_kind=kind)
    assert st == 0
    grid = oracle.grid_values().astype(np.float64)

    def small_bins(v):
        stat = oracle.norm_stat(v, kind) if scope == 0 else oracle.bucket_stat(v[:128], kind)
        n = float(oracle.norm_of(stat, kind))
        j = int(np.searchsorted(grid, float(v[1]) / n * (1 + 1e-9), side="right") - 1)
        # the layer-scope histogram bins by the centre of a raw-magnitude bin, which may sit one grid bin off
        return {j - 1, j, j + 1}, n

    wa, na = small_bins(a)
    wb, nb = small_bins(b)
    top = {255, 256}
    assert not (wa & wb) and not (wa & top) and not (wb & top)
    mass_a = sum(int(pooled[0][j]) for j in wa)
    mass_b = sum(int(pooled[0][j]) for j in wb)
    assert mass_a > 0 and mass_b > 0
    # integer weights floor(w * 2^(23 - e)): the smaller one has about 2^23 / ratio units, hence the tolerance
    assert mass_a / mass_b == pytest.approx((na / nb) ** 2, rel=2e-4)
    expected = {LINF: (1.0 / 2.0) ** 2, L1: ((1 + 127 * 0.25) / (2 + 127 * 0.002)) ** 2}[kind]   # per bucket or per layer alike
    assert (na / nb) ** 2 == pytest.approx(expected, rel=1e-5)
    assert np.all(np.diff(levs[0]) > 0) and levs[0][0] == 0 and levs[0][-1] == 1
