"""Pins for the pieces of the global-quantization / extra-gradient comparison (Sec. 4, Remark after eq. (MQV)):
the plain step against the closed form of extra-gradient on a bilinear game (contraction per singular value, while
a single gradient step expands), and "layer-wise is never worse than global" on the exact variance eq. (Var)."""
import numpy as np
import pytest

from paper_2505_14371_amd import workloads

LAYER, VECTOR = 0, 1


def test_extra_gradient_contracts_on_the_bilinear_game_and_a_single_step_expands(oracle):
    """F(z) = J z with J = [[0, A], [-A^T, 0]] (skew).  One extra-gradient round maps z to (I - gJ + g^2 J^2) z, whose
    singular values are sqrt(1 - g^2 s^2 + g^4 s^4) < 1 for g s < 1; one plain step maps z to (I - gJ) z, which expands
    by sqrt(1 + g^2 s^2).  The oracle's step is applied to the exact operator (no quantization) and compared with the
    float64 matrix form."""
    n = 64
    A, x0, y0 = workloads.bilinear_game(seed=3, n=n)
    A64 = A.astype(np.float64)
    J = np.block([[np.zeros((n, n)), A64], [-A64.T, np.zeros((n, n))]])
    gamma = np.float32(0.5 / np.linalg.norm(A64, 2))
    z = np.concatenate([x0, y0]).astype(np.float32)
    F = lambda v: (J @ v.astype(np.float64)).astype(np.float32)
    T = np.eye(2 * n) - float(gamma) * J + float(gamma) ** 2 * (J @ J)
    want = z.astype(np.float64)
    norms = [np.linalg.norm(z)]
    for _ in range(30):
        half = oracle.extrapolate(F(z), z, gamma)          # X_{t+1/2} = X_t - g F(X_t)
        z = oracle.extrapolate(F(half), z, gamma)          # X_{t+1}   = X_t - g F(X_{t+1/2})
        want = T @ want
        norms.append(np.linalg.norm(z))
        assert np.allclose(z, want, rtol=0, atol=2e-4 * norms[0])
    assert all(b < a for a, b in zip(norms, norms[1:]))
    sv = np.linalg.svd(A64, compute_uv=False)
    worst = np.sqrt(1 - (gamma * sv.min()) ** 2 + (gamma * sv.min()) ** 4)
    assert norms[-1] <= norms[0] * worst ** 30 * (1 + 1e-3)
    one = oracle.extrapolate(F(z), z, gamma)               # a single step on its own expands
    assert np.linalg.norm(one) > np.linalg.norm(z)
    assert np.array_equal(oracle.extrapolate(np.zeros(5, np.float32), np.arange(5, dtype=np.float32), 0.3),
                          np.arange(5, dtype=np.float32))


def exact_variance(g_layers, norms, levels):
    """eq. (Var): sum over layers of norm^2 sum_i (l_{tau+1} - u_i)(u_i - l_tau), float64."""
    tot = 0.0
    for v, n, lev in zip(g_layers, norms, levels):
        if n == 0:
            continue
        lev = np.asarray(lev, np.float64)
        u = np.minimum(np.abs(v.astype(np.float64)) / n, 1.0)
        tau = np.clip(np.searchsorted(lev, u, side="right") - 1, 0, lev.size - 2)
        tot += n ** 2 * float(np.sum((lev[tau + 1] - u) * (u - lev[tau])))
    return tot


def test_layerwise_quantization_is_not_worse_than_global(oracle):
    """Remark after eq. (MQV).  Layers of very different scale (the regime the paper argues from): per-layer norms
    with one fitted sequence per layer against one norm for the whole vector with one fitted sequence."""
    S, K = 8, 2
    w = workloads.mini("dcgan", max_layer=30000, max_layers=6)
    L = len(w.sizes)
    g = [workloads.node_numpy(w, k, 1) for k in range(K)]
    flat = [g[k][l] for k in range(K) for l in range(L)]
    uni = (np.arange(S) / (S - 1)).astype(np.float32)
    lw, _, _, _ = oracle.fit_levels(w.sizes, list(range(L)), [S] * L, K, flat, [uni] * L, scope=LAYER)
    gl, _, _, _ = oracle.fit_levels(w.sizes, [0] * L, [S], K, flat, [uni], scope=VECTOR)
    var_lw = var_gl = var_gl_uniform = 0.0
    for k in range(K):
        ln = [float(np.sqrt(np.sum(a.astype(np.float64) ** 2))) for a in g[k]]
        vn = float(np.sqrt(sum(x * x for x in ln)))
        var_lw += exact_variance(g[k], ln, lw)
        var_gl += exact_variance(g[k], [vn] * L, [gl[0]] * L)
        var_gl_uniform += exact_variance(g[k], [vn] * L, [uni] * L)
    assert var_lw < var_gl < var_gl_uniform
    assert var_lw < 0.8 * var_gl                      # heterogeneous layers: a clear gap, not a tie (about 0.68 here)
