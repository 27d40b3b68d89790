"""The torch-facing loop (paper_2505_14371_amd.solver.QODA: buffers and marshalling only) against the oracle's
free-running Alg. 1 on the bilinear game: the parameters it leaves are the query points X_{t+1/2}, bit for bit."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import helpers  # noqa: E402
from paper_2505_14371_amd import qoda, workloads  # noqa: E402
from paper_2505_14371_amd.solver import QODA  # noqa: E402


def _need_gpu():
    if not torch.cuda.is_available():
        pytest.fail("a GPU test was selected but no GPU is visible")


@pytest.mark.parametrize("q_hat", [None, 0.25])
def test_bilinear_game_through_the_solver_loop(oracle, q_hat):
    _need_gpu()
    dev = torch.device("cuda:0")
    wl = workloads.get("bilinear")
    A, x0, y0 = workloads.bilinear_game(seed=wl.seed)
    op = lambda x, y, k, t: workloads.bilinear_operator(A, x, y, k, t, seed=wl.seed, sigma=0.1)
    n, K, S = 512, wl.num_nodes, wl.points
    px = torch.from_numpy(x0.copy()).to(dev)
    py = torch.from_numpy(y0.copy()).to(dev)
    opt = QODA([px, py], num_nodes=K, points=S, seed=wl.seed, q_hat=q_hat, keep_next=True)
    lev = helpers.uniform_levels(S)
    ref = helpers.OracleQODA([n, n], [S, S], [lev, lev], K, [x0, y0], wl.seed, q_hat=q_hat)
    for t in range(1, 61):
        xq, yq = px.cpu().numpy(), py.cpu().numpy()
        assert np.array_equal(xq, ref.x_half[0]) and np.array_equal(yq, ref.x_half[1]), t
        host = [op(xq, yq, k, t) for k in range(K)]
        grads = [[torch.from_numpy(g).to(dev) for g in host[k]] for k in range(K)]
        opt.step(grads)
        ref.round_([list(h) for h in host], t)
        rates = opt.rates.cpu().numpy()
        assert rates[0] == ref.eta and rates[1] == (ref.gamma if q_hat is not None else ref.eta), t
    xn = [x.cpu().numpy() for x in opt.state_point()]
    assert np.array_equal(xn[0], ref.x_next[0]) and np.array_equal(xn[1], ref.x_next[1])
    assert opt.status() == qoda.OK
    opt.close()


def test_refits_at_the_update_steps(oracle):
    """fit_every = 2: levels are refitted at rounds 1, 3, 5 from that round's vectors (the set U of Alg. 1); two
    tensor kinds get the two default types."""
    _need_gpu()
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(2)
    shapes = [(40, 30), (30,), (30, 50), (50,)]
    K, S = 3, 8
    params = [torch.from_numpy(rng.standard_normal(s).astype(np.float32)).to(dev) for s in shapes]
    x1 = [p.cpu().numpy().ravel().copy() for p in params]
    opt = QODA(params, num_nodes=K, points=S, seed=5, fit_every=2)
    sizes = [int(np.prod(s)) for s in shapes]
    types = [0, 1, 0, 1]
    levels = [helpers.uniform_levels(S), helpers.uniform_levels(S)]
    y = [np.zeros(d, np.float32) for d in sizes]
    prev = [None] * K
    acc = 0.0
    for t in range(1, 6):
        host = [[(rng.standard_t(4, d) * 0.1 * (l + 1)).astype(np.float32) for l, d in enumerate(sizes)] for _ in range(K)]
        opt.step([[torch.from_numpy(g.reshape(shapes[l])).to(dev) for l, g in enumerate(host[k])] for k in range(K)])
        if (t - 1) % 2 == 0:
            flat = [host[k][l] for k in range(K) for l in range(len(sizes))]
            levels, _, _, st = oracle.fit_levels(sizes, types, [S, S], K, flat, levels)
            assert st == 0
        for ty in range(2):
            assert np.array_equal(opt.ctx.get_levels(ty), levels[ty]), (t, ty)
        lev_l = [levels[ty] for ty in types]
        msgs, deltas = [], []
        for k in range(K):
            m, _, dl, st = oracle.quantize(sizes, [S] * 4, lev_l, host[k], 5, t, k, msg_prev=prev[k])
            msgs.append(m)
            deltas.append(dl)
        prev = msgs
        mean = oracle.dequant_aggregate(sizes, [S] * 4, msgs)
        acc, eta = oracle.step_size(deltas, acc)
        for l in range(4):
            _, xh = oracle.oda_update(mean[l], x1[l], y[l], eta, eta)
            assert np.array_equal(params[l].cpu().numpy().ravel(), xh), (t, l)
    opt.close()


def test_argument_checks():
    _need_gpu()
    dev = torch.device("cuda:0")
    p = torch.zeros(100, device=dev)
    with pytest.raises(ValueError):
        QODA([p.double()], num_nodes=2)
    with pytest.raises(ValueError):
        QODA([], num_nodes=2)
    opt = QODA([p], num_nodes=2)
    with pytest.raises(ValueError):
        opt.step([[torch.zeros(100, device=dev)]])                 # one list for two nodes
    with pytest.raises(ValueError):
        opt.step([[torch.zeros(99, device=dev)], [torch.zeros(100, device=dev)]])
    with pytest.raises(RuntimeError):
        opt.state_point()
    opt.close()
