"""Pins for the oracle's level fit (Sec. 3.2, eq. (Qada2) with the weights lambda_z).  The paper states the
objective and leaves the optimiser to third-party code it does not describe, so what is pinned is that the
fit minimises that objective on its histogram grid: brute force on tiny cases, the uniform-density closed
form (equal gaps, from the stationarity condition of eq. (Qada2)), "layer-wise is never worse than global"
(Remark after eq. (MQV)), scale invariance and norm^2 weighting."""
import itertools

import numpy as np
import pytest

from paper_2505_14371_amd import workloads


def objective(W, lev):
    """sum_j W_j (l_{tau+1} - m_j)(m_j - l_tau) over grid bins below 1, from the definition (float64)."""
    import oracle

    mids = oracle.grid_mids()[:-1]
    lev = np.asarray(lev, dtype=np.float64)
    tau = np.clip(np.searchsorted(lev, mids, side="right") - 1, 0, len(lev) - 2)
    return float(np.sum(np.asarray(W[:-1], dtype=np.float64) * (lev[tau + 1] - mids) * (mids - lev[tau])))


def test_histogram_counts_magnitude_bit_patterns(oracle):
    v = workloads.layer_numpy(workloads.get("dcgan"), 0, 4, 1)
    v[:5] = [0.0, -0.0, np.inf, -1.0, 2.0 ** -130]
    h = oracle.histogram(v)                                          # every coordinate counts (Alg. 1 line 4)
    want = np.bincount((v.view(np.uint32) & 0x7FFFFFFF) >> 20, minlength=2048)
    assert np.array_equal(h, want) and h.sum() == v.size
    assert np.array_equal(oracle.histogram(v[:200]), np.bincount((v[:200].view(np.uint32) & 0x7FFFFFFF) >> 20, minlength=2048))


def test_grid_is_three_mantissa_bits_per_octave(oracle):
    g = oracle.grid_values().astype(np.float64)
    assert g[0] == 2.0 ** -32 and g[-1] == 1.0 and g.size == 257
    assert np.allclose(g[8:] / g[:-8], 2.0)
    assert np.allclose(g[1:9] / g[0], 1 + np.arange(1, 9) / 8)
    m = oracle.grid_mids()
    assert np.allclose(m[:-1], (g[:-1] + g[1:]) / 2) and m[-1] == 1.0


@pytest.mark.parametrize("S", [3, 4])
def test_dp_equals_brute_force_on_small_supports(oracle, S):
    rng = np.random.default_rng(S)
    g = oracle.grid_values()
    for trial in range(4):
        W = np.zeros(257, dtype=np.uint64)
        support = rng.choice(np.arange(200, 256), size=12, replace=False)
        W[support] = rng.integers(1, 1000, support.size).astype(np.uint64)
        lev = oracle.fit_dp(W, S)
        assert lev[0] == 0 and lev[-1] == 1 and np.all(np.diff(lev) > 0)
        assert set(lev[1:-1].tolist()) <= set(g.tolist())
        got = objective(W, lev)
        assert got == pytest.approx(oracle.fit_objective(W, lev), rel=1e-12, abs=1e-9)
        best = min(objective(W, np.concatenate([[0.0], g[list(c)], [1.0]]))
                   for c in itertools.combinations(range(180, 256), S - 2))
        assert got == pytest.approx(best, rel=1e-9)


def test_dp_is_never_worse_than_other_level_sets_on_the_grid(oracle):
    rng = np.random.default_rng(21)
    g = oracle.grid_values()
    v = np.abs(workloads.layer_numpy(workloads.get("txl"), 0, 3, 1))
    lev_in = [np.array([0, 1], np.float32)]
    for S in (4, 8, 16):
        levs, hist, pooled, st = oracle.fit_levels([v.size], [0], [S], 1, [v], [np.zeros(S, np.float32)])
        lev, W = levs[0], pooled[0]
        assert st == 0 and np.all(np.diff(lev) > 0) and lev[0] == 0 and lev[-1] == 1
        f = objective(W, lev)
        uni = np.concatenate([[0.0], g[np.searchsorted(g, np.arange(1, S - 1) / (S - 1))], [1.0]])
        assert f <= objective(W, uni)
        for _ in range(200):
            c = np.sort(rng.choice(np.arange(1, 256), S - 2, replace=False))
            assert f <= objective(W, np.concatenate([[0.0], g[c], [1.0]])) * (1 + 1e-12)
        # moving any single level to a neighbouring grid point does not help (coordinate-wise optimality, which
        # is the discrete form of the stationarity condition of eq. (Qada2))
        idx = np.searchsorted(g, lev[1:-1])
        for j in range(S - 2):
            for step in (-1, 1):
                c = idx.copy()
                c[j] += step
                if c[j] < 1 or c[j] > 255 or len(set(c.tolist())) < S - 2 or np.any(np.diff(c) <= 0):
                    continue
                assert f <= objective(W, np.concatenate([[0.0], g[c], [1.0]])) * (1 + 1e-12)
    del lev_in


def test_uniform_density_gives_equal_gaps(oracle):
    """For a uniform density on [0, 1] the stationarity condition of eq. (Qada2),
    int_{l_{j-1}}^{l_j} (u - l_{j-1}) dF = int_{l_j}^{l_{j+1}} (l_{j+1} - u) dF, forces equal gaps.  On the
    histogram grid the fitted levels therefore sit within one grid step (1/8 relative) of j/(S-1)."""
    g = oracle.grid_values().astype(np.float64)
    width = np.diff(g)
    W = np.zeros(257, dtype=np.uint64)
    W[:-1] = np.round(width * 2.0 ** 40).astype(np.uint64)
    for S in (3, 5, 9):
        lev = oracle.fit_dp(W, S).astype(np.float64)
        want = np.arange(S) / (S - 1)
        assert np.all(np.abs(lev[1:-1] - want[1:-1]) <= want[1:-1] / 8 + 1e-12), (S, lev)


def test_fit_is_scale_invariant_and_weights_nodes_by_squared_norm(oracle):
    w = workloads.mini("dcgan", max_layer=30000, max_layers=2)
    K = 2
    grads = [workloads.layer_numpy(w, k, l, 1) for k in range(K) for l in range(2)]
    zero = [np.zeros(8, np.float32)] * 2
    levs, hist, pooled, st = oracle.fit_levels(w.sizes, [0, 1], [8, 8], K, grads, zero)
    # multiplying every vector by a power of two changes nothing (levels live on normalised coordinates)
    levs2, _, pooled2, _ = oracle.fit_levels(w.sizes, [0, 1], [8, 8], K, [g * np.float32(64.0) for g in grads], zero)
    assert all(np.array_equal(a, b) for a, b in zip(levs, levs2)) and np.array_equal(pooled, pooled2)
    # scaling ONE node by 4 multiplies its weight by 16 relative to the other node (lambda_z ~ ||g_z||^2)
    only0 = [grads[0], grads[1], np.zeros_like(grads[2]), np.zeros_like(grads[3])]
    only1 = [np.zeros_like(grads[0]), np.zeros_like(grads[1]), grads[2], grads[3]]
    _, _, p0, _ = oracle.fit_levels(w.sizes, [0, 1], [8, 8], K, only0, zero)
    _, _, p1, _ = oracle.fit_levels(w.sizes, [0, 1], [8, 8], K, only1, zero)
    s0, s1 = oracle.sumsq(grads[0]), oracle.sumsq(grads[2])
    both = pooled[0].astype(np.float64)
    # pooled = wfix0 * shape0 + wfix1 * shape1 with wfix proportional to the squared norms
    shape0 = p0[0].astype(np.float64) / p0[0].sum() * w.sizes[0]
    shape1 = p1[0].astype(np.float64) / p1[0].sum() * w.sizes[0]
    mix = (s0 * shape0 + s1 * shape1)
    assert np.allclose(both / both.sum(), mix / mix.sum(), rtol=1e-5, atol=1e-9)
    # pooled mass equals the number of non-zero-bin coordinates times the fixed-point weights
    assert int(hist.sum()) == K * sum(w.sizes)


def test_layerwise_fit_is_never_worse_than_one_shared_sequence(oracle):
    """Remark after eq. (MQV): optimising one sequence per type can only lower the objective."""
    w = workloads.mini("txl", max_layer=30000, max_layers=4)
    K = 2
    L = len(w.sizes)
    grads = [workloads.layer_numpy(w, k, l, 1) * np.float32(10.0 ** l) for k in range(K) for l in range(L)]
    S = 8
    per, _, pooled_per, _ = oracle.fit_levels(w.sizes, list(range(L)), [S] * L, K, grads, [np.zeros(S, np.float32)] * L)
    glob, _, pooled_glob, _ = oracle.fit_levels(w.sizes, [0] * L, [S], K, grads, [np.zeros(S, np.float32)])
    layerwise = sum(objective(pooled_per[l], per[l]) for l in range(L))
    shared = sum(objective(pooled_per[l], glob[0]) for l in range(L))
    assert layerwise <= shared * (1 + 1e-12)


def test_all_zero_type_keeps_its_levels_and_nonfinite_is_flagged(oracle):
    keep = np.array([0, 0.2, 0.5, 1.0], np.float32)
    levs, _, pooled, st = oracle.fit_levels([100], [0], [4], 1, [np.zeros(100, np.float32)], [keep])
    assert st == 0 and np.array_equal(levs[0], keep) and pooled.sum() == 0
    bad = np.ones(100, np.float32)
    bad[3] = np.nan
    levs, _, _, st = oracle.fit_levels([100], [0], [4], 1, [bad], [keep])
    assert st == 1 and np.array_equal(levs[0], keep)


def test_fitted_levels_lower_the_real_quantization_variance(oracle):
    """End to end: on heavy-tailed vectors the fitted sequence gives a much smaller exact variance eq. (Var)
    than uniform levels with the same number of points."""
    w = workloads.get("dcgan")
    v = workloads.layer_numpy(w, 0, 3, 1)
    S = 16
    levs, _, _, _ = oracle.fit_levels([v.size], [0], [S], 1, [v], [np.zeros(S, np.float32)])
    norm, inv = oracle.norm_and_inv(v)
    u = np.minimum(np.abs(v.astype(np.float64)) / float(norm), 1.0)

    def var(lev):
        lev = lev.astype(np.float64)
        tau = np.clip(np.searchsorted(lev, u, side="right") - 1, 0, len(lev) - 2)
        return float(np.sum((lev[tau + 1] - u) * (u - lev[tau])))

    uni = (np.arange(S) / (S - 1)).astype(np.float32)
    assert var(levs[0]) < 0.05 * var(uni)
