"""GPU parity for the extra-gradient leg (qoda_extrapolate) and the global-quantization configuration (one norm for
the whole vector, one level sequence): an extra-gradient run on the bilinear game, two quantize + exchange +
step legs per round, GPU against the oracle's routines; and the layer-wise vs global error on the same kernels."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import helpers  # noqa: E402
from paper_2505_14371_amd import qoda, workloads  # noqa: E402


def gm(*a, **k):
    if not torch.cuda.is_available():
        pytest.fail("a GPU test was selected but no GPU is visible")
    import gpu_harness

    return gpu_harness.GpuModel(*a, **k)


@pytest.mark.parametrize("scope", [qoda.SCOPE_VECTOR, qoda.SCOPE_LAYER, qoda.SCOPE_BUCKET])
def test_extra_gradient_on_the_bilinear_game(oracle, scope):
    wl = workloads.get("bilinear")
    A, x0, y0 = workloads.bilinear_game(seed=wl.seed)
    op = lambda x, y, k, t: workloads.bilinear_operator(A, x, y, k, t, seed=wl.seed, sigma=0.1)
    n, K, S = 512, wl.num_nodes, 64
    sizes = [n, n]
    m = gm(sizes, [0, 0], [S], K, seed=wl.seed, norm_scope=scope)
    lev = helpers.uniform_levels(S)
    gamma = np.float32(0.4 / np.linalg.norm(A.astype(np.float64), 2))
    gdev = torch.tensor([gamma], dtype=torch.float32, device=m.x1.device)
    m.set_layers(m.x1, [x0, y0])                       # X_t lives in x1, X_{t+1/2} in x_half
    xt = [x0.copy(), y0.copy()]
    start = np.linalg.norm(np.concatenate(xt))
    calls = 0
    for t in range(1, 41):
        for leg in (0, 1):
            q = xt if leg == 0 else half
            grads = [list(op(q[0], q[1], k, 2 * t + leg)) for k in range(K)]
            m.set_grads(grads)
            m.ctx.quantize_all(m.grad_ptrs(), 2 * t + leg, m.msg[0], None)
            calls += 1
            out = m.x_half if leg == 0 else m.x1
            m.ctx.extrapolate(m.msg[0], m.layer_ptrs(m.x1), m.layer_ptrs(out), gdev)
            msgs = [oracle.quantize(sizes, [S, S], [lev, lev], grads[k], wl.seed, 2 * t + leg, k, scope=scope)[0]
                    for k in range(K)]
            got = m.messages(0)
            assert all(np.array_equal(a, b) for a, b in zip(got, msgs)), (t, leg)
            mean = oracle.dequant_aggregate(sizes, [S, S], msgs, scope=scope)
            new = [oracle.extrapolate(mean[l], xt[l], gamma) for l in range(2)]
            res = m.layers(out)
            assert all(np.array_equal(a, b) for a, b in zip(res, new)), (t, leg)
            if leg == 0:
                half = new
            else:
                xt = new
    assert calls == 80                                  # two exchanges per round, against one for QODA
    assert np.linalg.norm(np.concatenate(xt)) < 0.8 * start


def test_layerwise_error_is_below_global_on_the_same_kernels(oracle):
    """Aggregated quantization error ||mean_k Vhat_k - mean_k V_k||^2 with per-layer norms and one fitted sequence per
    layer, against one norm per node and one fitted sequence (Remark after eq. (MQV)); 8 grid points."""
    w = workloads.mini("dcgan", max_layer=200000, max_layers=10)
    L, K, S = len(w.sizes), 4, 8
    g = [workloads.node_numpy(w, k, 1) for k in range(K)]
    true_mean = [np.mean([g[k][l].astype(np.float64) for k in range(K)], axis=0) for l in range(L)]
    err = {}
    for name, types, pts, scope in (("layerwise", list(range(L)), [S] * L, qoda.SCOPE_LAYER),
                                    ("global", [0] * L, [S], qoda.SCOPE_VECTOR)):
        tot = 0.0
        for seed in range(3):
            m = gm(w.sizes, types, pts, K, seed=seed, norm_scope=scope)
            m.set_grads(g)
            m.fit(1)
            m.quantize_all(1)
            m.aggregate()
            mean = m.layers(m.mean)
            tot += sum(float(np.sum((mean[l].astype(np.float64) - true_mean[l]) ** 2)) for l in range(L))
        err[name] = tot / 3
    assert err["layerwise"] < 0.9 * err["global"], err     # about 0.8 on these vectors
