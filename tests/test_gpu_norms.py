"""GPU parity for the L1 and L-infinity normalisations (Sec. 2.2: the quantizer is defined for an L^q norm) in all three
norm scopes: statistics, norms, fitted levels, packed bytes, step-size terms and iterates against the oracle, bit for
bit; the statistics-based fit of bucket scope; non-finite input."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import helpers  # noqa: E402
from paper_2505_14371_amd import qoda, workloads  # noqa: E402

LAYER, VECTOR, BUCKET = qoda.SCOPE_LAYER, qoda.SCOPE_VECTOR, qoda.SCOPE_BUCKET
L1, LINF = qoda.NORM_L1, qoda.NORM_LINF


def gm(*a, **k):
    if not torch.cuda.is_available():
        pytest.fail("a GPU test was selected but no GPU is visible")
    import gpu_harness

    return gpu_harness.GpuModel(*a, **k)


RAGGED = [1, 3, 255, 257, 4100, 16383, 16385, 70000, 16384 * 3 + 7, 0, 16384 * 257 + 13]


@pytest.mark.parametrize("kind", [L1, LINF])
def test_statistics_and_norms_are_bit_exact(oracle, kind):
    K = 2
    m = gm(RAGGED, [0] * len(RAGGED), [4], K, seed=1, norm_kind=kind)
    rng = np.random.default_rng(kind)
    grads = [[(rng.standard_t(3, s) * 10.0 ** rng.uniform(-6, 3)).astype(np.float32) for s in RAGGED] for _ in range(K)]
    grads[1][3][:] = 0.0
    grads[0][4][:] = np.float32(1e-42)                                   # subnormal entries
    m.set_grads(grads)
    m.quantize_all(1)
    ss = m.ctx.read_buffer(qoda.BUF_SUMSQ)
    nr = m.ctx.read_buffer(qoda.BUF_NORM)
    iv = m.ctx.read_buffer(qoda.BUF_INV)
    assert m.ctx.status() == qoda.ETINYNORM                              # the subnormal layer: its norm is below 2^-126
    for k in range(K):
        for l, s in enumerate(RAGGED):
            want = oracle.norm_stat(grads[k][l], kind)
            assert ss[k, l] == want, (k, l, s)
            n = oracle.norm_of(want, kind)
            assert nr[k, l] == n and iv[k, l] == oracle.rcp_floor(n), (k, l)


@pytest.mark.parametrize("kind", [L1, LINF])
@pytest.mark.parametrize("scope", [LAYER, VECTOR, BUCKET])
@pytest.mark.parametrize("S", [2, 5, 16, 256])
def test_messages_match_for_every_scope(oracle, kind, scope, S):
    sizes = [3000, 257, 0, 16384 + 2048 * 3 + 19, 1]
    L, K = len(sizes), 2
    rng = np.random.default_rng(S)
    lev = helpers.uniform_levels(S)
    m = gm(sizes, [0] * L, [S], K, seed=31, norm_scope=scope, norm_kind=kind)
    grads = [[(rng.standard_t(4, s) * 10.0 ** rng.uniform(-3, 2)).astype(np.float32) for s in sizes] for _ in range(K)]
    m.set_grads(grads)
    m.quantize_all(1)
    msgs = m.messages()
    delta = m.ctx.read_buffer(qoda.BUF_DELTA)
    want = []
    for k in range(K):
        wm, _, dl, st = oracle.quantize(sizes, [S] * L, [lev] * L, grads[k], 31, 1, k, scope=scope, norm_kind=kind)
        assert st == 0
        assert np.array_equal(msgs[k], wm), k
        assert delta[k] == dl, k
        want.append(wm)
    m.aggregate()
    mean = m.layers(m.mean)
    ref = oracle.dequant_aggregate(sizes, [S] * L, want, scope=scope)
    for l in range(L):
        assert np.array_equal(mean[l], ref[l]), l
    assert m.ctx.status() == qoda.OK


@pytest.mark.parametrize("kind", [L1, LINF])
@pytest.mark.parametrize("scope", [LAYER, VECTOR, BUCKET])
def test_rounds_with_fit_previous_message_and_update(oracle, kind, scope):
    w = workloads.mini("txl", max_layer=50000, max_layers=6)
    sizes = list(w.sizes) + [16384 * 2 + 300, 0, 77]
    L, K, S = len(sizes), 3, 8
    types = [l % 3 for l in range(L)]
    rng = np.random.default_rng(3 + kind)
    x1 = [rng.standard_normal(s).astype(np.float32) for s in sizes]
    m = gm(sizes, types, [S, S, S], K, seed=4, norm_scope=scope, norm_kind=kind)
    m.set_layers(m.x1, x1)
    levels = [helpers.uniform_levels(S) for _ in range(3)]
    y = [np.zeros(s, np.float32) for s in sizes]
    prev = [None] * K
    acc = 0.0
    for t in range(1, 4):
        grads = [[(rng.standard_t(4, s) * 10.0 ** rng.uniform(-3, 1)).astype(np.float32) for s in sizes] for _ in range(K)]
        m.set_grads(grads)
        m.fit(t)
        flat = [grads[k][l] for k in range(K) for l in range(L)]
        levels, hist, pooled, st = oracle.fit_levels(sizes, types, [S] * 3, K, flat, levels, scope=scope, norm_kind=kind)
        assert st == 0
        assert np.array_equal(m.ctx.read_buffer(qoda.BUF_POOLED), pooled), t
        for ty in range(3):
            assert np.array_equal(m.ctx.get_levels(ty), levels[ty]), (t, ty)
        m.quantize_all(t)
        msgs = m.messages()
        delta = m.ctx.read_buffer(qoda.BUF_DELTA)
        lev_l = [levels[types[l]] for l in range(L)]
        want_msgs, want_delta = [], []
        for k in range(K):
            wm, _, dl, st = oracle.quantize(sizes, [S] * L, lev_l, grads[k], 4, t, k, msg_prev=prev[k], scope=scope,
                                            norm_kind=kind)
            assert np.array_equal(msgs[k], wm), (t, k)
            assert delta[k] == dl, (t, k)
            want_msgs.append(wm)
            want_delta.append(dl)
        prev = want_msgs
        mean = oracle.dequant_aggregate(sizes, [S] * L, want_msgs, scope=scope)
        acc, eta = oracle.step_size(want_delta, acc)
        m.step()
        assert float(m.acc.cpu()[0]) == acc and float(m.eta.cpu()[0]) == float(eta)
        gy, gxh, gxn = m.layers(m.y), m.layers(m.x_half), m.layers(m.x_next)
        for l in range(L):
            xn, xh = oracle.oda_update(mean[l], x1[l], y[l], eta, eta)
            assert np.array_equal(gy[l], y[l]) and np.array_equal(gxh[l], xh) and np.array_equal(gxn[l], xn), (t, l)
    assert m.ctx.status() == qoda.OK


@pytest.mark.parametrize("kind", [L1, LINF])
def test_fit_from_gathered_statistics(oracle, kind):
    """Bucket scope, fits from the statistics of the previous round's quantize pass (explicit fit in round 1)."""
    sizes = [5000, 1300, 0, 70000, 16384 * 5 + 77, 3]
    types = [0, 0, 1, 1, 2, 2]
    L, K, S, M = len(sizes), 3, 8, 3
    m = gm(sizes, types, [S] * M, K, seed=12, norm_scope=BUCKET, norm_kind=kind)
    rng = np.random.default_rng(5)
    levels = [helpers.uniform_levels(S) for _ in range(M)]
    prev = [None] * K
    exps = hist = bmax = None
    for t in range(1, 5):
        grads = [[(rng.standard_t(3, s) * 3.0 ** t * 10.0 ** rng.uniform(-3, 0)).astype(np.float32) for s in sizes]
                 for _ in range(K)]
        m.set_grads(grads)
        if t == 1:
            m.fit(1)
            flat = [grads[k][l] for k in range(K) for l in range(L)]
            levels, _, pooled, st = oracle.fit_levels(sizes, types, [S] * M, K, flat, levels, scope=BUCKET, norm_kind=kind)
            b0 = np.stack([oracle.quantize(sizes, [S] * L, [levels[ty] for ty in types], grads[k], 12, 0, k, scope=BUCKET,
                                           stats_exp=[oracle.TYPE_SKIP] * L, norm_kind=kind)[5] for k in range(K)])
            _, _, exps, _ = oracle.fit_from_stats(types, [S] * M, K, np.zeros((K, L, 257), np.uint64), b0,
                                                  [oracle.TYPE_SKIP] * M, levels, norm_kind=kind)
        else:
            m.ctx.fit_levels(None, t)
            levels, pooled, exps, st = oracle.fit_from_stats(types, [S] * M, K, hist, bmax, exps, levels, norm_kind=kind)
        assert st == 0
        assert np.array_equal(m.ctx.read_buffer(qoda.BUF_POOLED), pooled), t
        for ty in range(M):
            assert np.array_equal(m.ctx.get_levels(ty), levels[ty]), (t, ty)
        m.quantize_all(t)
        msgs = m.messages()
        lev_l = [levels[ty] for ty in types]
        hist = np.zeros((K, L, 257), np.uint64)
        bmax = np.zeros((K, L))
        want = []
        for k in range(K):
            out = oracle.quantize(sizes, [S] * L, lev_l, grads[k], 12, t, k, msg_prev=prev[k], scope=BUCKET,
                                  stats_exp=[int(exps[ty]) for ty in types], norm_kind=kind)
            assert np.array_equal(msgs[k], out[0]), (t, k)
            hist[k], bmax[k] = out[4], out[5]
            want.append(out[0])
        prev = want
        m.step()
    assert not np.array_equal(levels[0], helpers.uniform_levels(S))


@pytest.mark.parametrize("kind", [L1, LINF])
@pytest.mark.parametrize("scope", [LAYER, VECTOR, BUCKET])
def test_nonfinite_input_is_flagged(kind, scope):
    for bad in (np.inf, np.nan):
        m = gm([1000, 300], [0, 0], [4], 1, seed=1, norm_scope=scope, norm_kind=kind)
        g = [[np.ones(1000, np.float32), np.ones(300, np.float32)]]
        g[0][0][300] = bad
        m.set_grads(g)
        m.quantize_all(1)
        assert m.ctx.status() == qoda.ENONFINITE
        assert m.ctx.status() == qoda.OK


def test_unknown_norm_kind_is_rejected():
    if not torch.cuda.is_available():
        pytest.fail("a GPU test was selected but no GPU is visible")
    with pytest.raises(qoda.QodaError):
        qoda.Context([10], [0], [4], 1, 0, norm_kind=3)
