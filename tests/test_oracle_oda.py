"""Pins for the oracle's optimistic dual averaging update and adaptive step size (Sec. 4: eq. (ODA),
eq. (general_stepsize), Alg. 1) -- first-round special case, the closed form of X_t used in the analysis
(App. E), the no-quantization limit, and convergence on the bilinear saddle game."""
import math

import numpy as np
import pytest

import helpers
from paper_2505_14371_amd import workloads


def test_step_size_formula_and_first_round(oracle):
    # eta_1 = gamma_1 = 1 (empty sum); then (1 + sum_s sum_k ||.||^2 / K^2)^(-1/2)
    acc, eta = oracle.step_size([0.0, 0.0], 0.0)
    assert acc == 0.0 and float(eta) == 1.0
    acc, eta = oracle.step_size([3.0, 5.0, 4.0], 0.0)          # K = 3: 12 / 9
    assert acc == pytest.approx(12.0 / 9.0, rel=1e-15)
    assert float(eta) == pytest.approx((1 + 12.0 / 9.0) ** -0.5, rel=3e-7)
    acc2, eta2 = oracle.step_size([1.0, 1.0, 1.0], acc)
    assert acc2 == pytest.approx(15.0 / 9.0, rel=1e-15)
    assert float(eta2) < float(eta)                              # non-increasing
    rng = np.random.default_rng(0)
    a = 0.0
    last = 1.0
    for _ in range(200):
        a, e = oracle.step_size(rng.uniform(0, 10, 4), a)
        assert 0 < float(e) <= last
        assert float(e) == pytest.approx((1 + a) ** -0.5, rel=3e-7)
        last = float(e)


def test_oda_update_matches_the_equations(oracle):
    rng = np.random.default_rng(3)
    n = 1000
    mean, x1, y = (rng.standard_normal(n).astype(np.float32) for _ in range(3))
    y0 = y.copy()
    xn, xh = oracle.oda_update(mean, x1, y, 0.37, 0.37)
    y_ref = y0.astype(np.float64) - mean
    assert np.allclose(y, y_ref, rtol=1e-6, atol=1e-6)
    assert np.allclose(xn, x1 + 0.37 * y_ref, rtol=1e-6, atol=1e-6)             # X_{t+1} = X_1 + eta Y_{t+1}
    assert np.allclose(xh, x1 + 0.37 * y_ref - 0.37 * mean, rtol=1e-6, atol=1e-6)  # X_{t+3/2} = X_{t+1} - gamma mean
    # a sign error on either term would be far outside the tolerance
    assert not np.allclose(xh, x1 + 0.37 * y_ref + 0.37 * mean, rtol=1e-3, atol=1e-3)


def test_closed_form_of_the_iterates_every_round(oracle):
    """App. E: X_t = X_1 - (eta_t / K) sum_{s<t} sum_k Vhat_{k,s+1/2}; Y is the running sum of the means."""
    w = workloads.mini("dcgan", max_layer=2500, max_layers=3)
    K = 3
    points = [8, 16, 4]
    levels = [helpers.uniform_levels(S) for S in points]
    rng = np.random.default_rng(1)
    x1 = [rng.standard_normal(s).astype(np.float32) for s in w.sizes]
    st = helpers.OracleQODA(w.sizes, points, levels, K, x1, seed=11)
    run_sum = [np.zeros(s) for s in w.sizes]
    for t in range(1, 7):
        grads = [workloads.node_numpy(w, k, t) for k in range(K)]
        msgs, deltas, mean = st.round_(grads, t)
        dec = [oracle.dequant_aggregate(w.sizes, points, [m]) for m in msgs]
        for l in range(len(w.sizes)):
            run_sum[l] += np.mean([dec[k][l].astype(np.float64) for k in range(K)], axis=0)
            scale = np.abs(run_sum[l]).max() + 1e-30
            assert np.allclose(st.y[l], -run_sum[l], rtol=0, atol=2e-6 * scale)
            assert np.allclose(st.x_next[l] - x1[l].astype(np.float64), float(st.eta) * st.y[l].astype(np.float64),
                               rtol=0, atol=2e-6 * (np.abs(x1[l]).max() + scale))
        if t == 1:
            # first round: no previous messages, so delta_k = ||Vhat_k||^2
            for k in range(K):
                assert deltas[k] == pytest.approx(sum(float(np.sum(dec[k][l].astype(np.float64) ** 2))
                                                      for l in range(len(w.sizes))), rel=1e-5)


def test_fine_levels_approach_unquantized_dual_averaging(oracle):
    """With 256 uniform levels the quantization error is tiny, so the trajectory stays close to eq. (ODA) run on
    the exact vectors in float64."""
    A, x0, y0 = workloads.bilinear_game(seed=0, n=64)
    op = lambda x, y, k, t: workloads.bilinear_operator(A, x, y, k, t, seed=0, sigma=0.1)
    q_fine, _ = helpers.run_bilinear(4, 30, 256, 0, op, x0, y0, quantize=True)
    q_coarse, _ = helpers.run_bilinear(4, 30, 4, 0, op, x0, y0, quantize=True)
    q_exact, _ = helpers.run_bilinear(4, 30, 256, 0, op, x0, y0, quantize=False)
    err_fine = max(np.linalg.norm(a - b) for a, b in zip(q_fine, q_exact))
    err_coarse = max(np.linalg.norm(a - b) for a, b in zip(q_coarse, q_exact))
    scale = np.linalg.norm(q_exact[0])
    assert err_fine < 0.03 * scale
    assert err_coarse > 3 * err_fine


def test_bilinear_game_ergodic_average_approaches_the_equilibrium(oracle):
    """Config 1: min_x max_y x^T A y, n = 512, K = 4, 8 uniform levels, 200 rounds; equilibrium 0.  The paper
    gives a rate (Thm 5.4: O(eps_Q-dependent constant / sqrt(TK))) but no constants, so the thresholds come from
    the unquantized run: the norm of the ergodic average of the query points X_{t+1/2} decreases with T, and the
    finer the levels (smaller eps_Q) the closer it gets to the unquantized value.  With 8 uniform levels at
    d = 512 the quantization variance is about 2.3 ||v||^2, the adaptive step size shrinks accordingly and
    progress is slow; a sign error in the update would make the norm grow instead."""
    wl = workloads.get("bilinear")
    A, x0, y0 = workloads.bilinear_game(seed=wl.seed)
    op = lambda x, y, k, t: workloads.bilinear_operator(A, x, y, k, t, seed=wl.seed, sigma=0.1)
    marks = (10, 50, 100, 200)
    avg = {}
    for S in (wl.points, 64):
        q, st = helpers.run_bilinear(wl.num_nodes, wl.rounds, S, wl.seed, op, x0, y0, quantize=True)
        avg[S] = [np.linalg.norm(np.mean(q[:T], axis=0)) for T in marks]
        assert 0 < float(st.eta) < 1
    e, _ = helpers.run_bilinear(wl.num_nodes, wl.rounds, wl.points, wl.seed, op, x0, y0, quantize=False)
    avg_e = [np.linalg.norm(np.mean(e[:T], axis=0)) for T in marks]
    start = np.linalg.norm(np.concatenate([x0, y0]))
    for a in (avg[wl.points], avg[64], avg_e):
        assert start > a[0] > a[1] > a[2] > a[3]
    assert avg_e[3] < 0.6 * start                                   # unquantized: 31.3 -> about 16.4
    assert avg_e[3] < avg[64][3] < avg[wl.points][3] < 0.985 * start
    assert avg[64][3] < 1.2 * avg_e[3]
